// Query / data preparation kernels: normalisation (cosine), rotation by the fixed orthogonal
// transform Q (Alg. 1 and Alg. 2, rotation step) and the projection tables
// (Alg. 2, projection-table step).  All sums are fp64 sums of exact fp32 x fp32 products,
// rounded once to fp32, so that they agree with a plain fp64 evaluation to the last bit in all
// but a vanishing fraction of the outputs.
#include <hipcub/hipcub.hpp>

#include <algorithm>
#include <string>

#include "pag_internal.h"

namespace {

typedef double double4_t __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------------------
// Rotation: OUT[i][j] = fl32( sum_k X[i][k] * R[j][k] ),  X [rows x d], R [d x d] row-major.
// The one dense contraction of the path: fp64 MFMA (v_mfma_f64_16x16x4), 64 x 64 output tile
// per workgroup of 4 waves, each wave a 32 x 32 sub-tile (2 x 2 MFMA tiles), K staged through
// LDS in steps of 32 as doubles.  Rows of the LDS tiles are padded to 36 doubles (72 dwords,
// = 8 mod 64 banks) so that the 16 rows x 4 k-columns read by one MFMA operand fetch spread
// over all banks.
// ---------------------------------------------------------------------------------------
constexpr int BM = 64, BN = 64, KT = 32, LDT = 36;

__global__ void __launch_bounds__(256) k_rotate(const float* __restrict__ X, u64 rows, u32 d,
                                                const float* __restrict__ R, float* __restrict__ OUT) {
    __shared__ double As[BM][LDT];
    __shared__ double Bs[BN][LDT];
    const int t = threadIdx.x, lane = t & 63, w = t >> 6;
    const int wm = w >> 1, wn = w & 1;
    const u64 m0 = (u64)blockIdx.y * BM;
    const u32 n0 = blockIdx.x * BN;
    double4_t acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = (double4_t){0.0, 0.0, 0.0, 0.0};

    for (u32 k0 = 0; k0 < d; k0 += KT) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int idx = t + 256 * i, row = idx >> 3, k4 = (idx & 7) * 4;
            float4 a = make_float4(0.f, 0.f, 0.f, 0.f), bb = a;
            if (m0 + row < rows && k0 + k4 < d) a = *(const float4*)(X + (m0 + row) * d + k0 + k4);
            if (n0 + row < d && k0 + k4 < d) bb = *(const float4*)(R + (u64)(n0 + row) * d + k0 + k4);
            As[row][k4 + 0] = (double)a.x; As[row][k4 + 1] = (double)a.y;
            As[row][k4 + 2] = (double)a.z; As[row][k4 + 3] = (double)a.w;
            Bs[row][k4 + 0] = (double)bb.x; Bs[row][k4 + 1] = (double)bb.y;
            Bs[row][k4 + 2] = (double)bb.z; Bs[row][k4 + 3] = (double)bb.w;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < KT; kk += 4) {
            const int r = lane & 15, kq = kk + (lane >> 4);
            const double a0 = As[wm * 32 + r][kq], a1 = As[wm * 32 + 16 + r][kq];
            const double b0 = Bs[wn * 32 + r][kq], b1 = Bs[wn * 32 + 16 + r][kq];
            acc[0][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b1, acc[1][1], 0, 0, 0);
        }
        __syncthreads();
    }
    // accumulator layout of the 16x16 f64 tile: register r of lane l holds row l/16 + 4*r, column l%16
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const u64 row = m0 + wm * 32 + i * 16 + (lane >> 4) + 4 * r;
                const u32 col = n0 + wn * 32 + j * 16 + (lane & 15);
                if (row < rows && col < d) OUT[row * d + col] = (float)acc[i][j][r];
            }
}

// tables[row][l][j] = fl32( sum_k r_jl[k] * q_l[k] ), k ascending; rows l >= P are zero padding.
__global__ void __launch_bounds__(256) k_tables(const float* __restrict__ qrot, u64 rows, u32 d, u32 P,
                                                u32 Ppad, u32 dsub, const float* __restrict__ cb,
                                                float* __restrict__ tables) {
    const u64 gid = (u64)blockIdx.x * 256 + threadIdx.x;
    const u64 per_row = (u64)Ppad * PAG_NCODE;
    if (gid >= rows * per_row) return;
    const u64 row = gid / per_row;
    const u32 lj = (u32)(gid % per_row), l = lj / PAG_NCODE;
    float out = 0.f;
    if (l < P) {
        const float* r = cb + (u64)lj * dsub;
        const float* q = qrot + row * d + (u64)l * dsub;
        double acc = 0.0;
        for (u32 k = 0; k < dsub; ++k) acc = __builtin_fma((double)r[k], (double)q[k], acc);
        out = (float)acc;
    }
    tables[gid] = out;
}

// out = x / ||x||, one wave per row; norm from an fp64 sum of squares.
__global__ void __launch_bounds__(64) k_normalise(const float* __restrict__ X, u64 rows, u32 d,
                                                  float* __restrict__ out) {
    const u64 row = blockIdx.x;
    if (row >= rows) return;
    const int lane = threadIdx.x;
    const float* x = X + row * d;
    double s = 0.0;
    for (u32 k = lane; k < d; k += 64) s = __builtin_fma((double)x[k], (double)x[k], s);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    double nrm = sqrt(s);
    if (nrm == 0.0) nrm = 1.0;
    for (u32 k = lane; k < d; k += 64) out[row * d + k] = (float)((double)x[k] / nrm);
}

// float -> __half (round to nearest even) or __half -> float (exact), one element per thread
__global__ void __launch_bounds__(256) k_convert(const void* __restrict__ src, u32 src_half, void* __restrict__ dst,
                                                 u32 dst_half, u64 count) {
    const u64 i = (u64)blockIdx.x * 256 + threadIdx.x;
    if (i >= count) return;
    const float v = src_half ? __half2float(((const __half*)src)[i]) : ((const float*)src)[i];
    if (dst_half) ((__half*)dst)[i] = __float2half_rn(v);
    else ((float*)dst)[i] = v;
}

__global__ void __launch_bounds__(256) k_zero_u32(u32* p, u64 count) {
    const u64 i = (u64)blockIdx.x * 256 + threadIdx.x;
    if (i < count) p[i] = 0u;
}

// ---------------------------------------------------------------------------------------
// Query order.  The waves take the queries of a batch a few thousand at a time; when the queries that run side by
// side search the same part of the graph, part of their rows comes from the memory-side cache instead of HBM.  The
// batch is therefore taken in the order of its projections onto its direction of largest spread, found by two steps
// of the power iteration from the best of ORDER_CAND stored vectors (the first entry nodes, i.e. random data
// points: the one along which the batch varies most).  Results do not depend on the order.
// ---------------------------------------------------------------------------------------
constexpr u32 ORDER_CAND = 16;

// dirs[k] = stored vector of entry[k] as fp32, norm2[k] = its squared length
__global__ void __launch_bounds__(64) k_order_dirs(pag_vecs vec, const u32* __restrict__ entry, float* __restrict__ dirs,
                                                   float* __restrict__ norm2) {
    const u32 k = blockIdx.x, d = vec.d;
    const u32 id = entry[k];
    float acc = 0.f;
    for (u32 c = threadIdx.x; c < d / 4; c += 64) {
        const float4 x = pag_vload4(vec, id, c);
        ((float4*)(dirs + (u64)k * d))[c] = x;
        acc += x.x * x.x + x.y * x.y + x.z * x.z + x.w * x.w;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
    if (threadIdx.x == 0) norm2[k] = acc;
}

// proj[row][k] = <q_row, dirs[k]>, one wave per row
__global__ void __launch_bounds__(64) k_order_project(const float* __restrict__ qrot, u64 rows, u32 d, const float* __restrict__ dirs,
                                                      u32 ncand, float* __restrict__ proj) {
    const u64 row = blockIdx.x;
    if (row >= rows) return;
    const int lane = threadIdx.x;
    float acc[ORDER_CAND];
#pragma unroll
    for (u32 k = 0; k < ORDER_CAND; ++k) acc[k] = 0.f;
    for (u32 c = lane; c < d / 4; c += 64) {
        const float4 q = ((const float4*)(qrot + row * d))[c];
#pragma unroll
        for (u32 k = 0; k < ORDER_CAND; ++k)
            if (k < ncand) {
                const float4 x = ((const float4*)(dirs + (u64)k * d))[c];
                acc[k] += q.x * x.x + q.y * x.y + q.z * x.z + q.w * x.w;
            }
    }
#pragma unroll
    for (u32 k = 0; k < ORDER_CAND; ++k) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) acc[k] += __shfl_xor(acc[k], o, 64);
        if ((u32)lane == k) proj[row * ORDER_CAND + k] = acc[k];
    }
}

// the candidate with the largest variance of the projections per unit length -> *best
__global__ void __launch_bounds__(1024) k_order_pick(const float* __restrict__ proj, u64 rows, u32 ncand, const float* __restrict__ norm2,
                                                     u32* __restrict__ best, float* __restrict__ pbar) {
    __shared__ double s1[1024], s2[1024];
    const u32 t = threadIdx.x, k = t % ORDER_CAND;
    double a = 0.0, b = 0.0;
    for (u64 r = t / ORDER_CAND; r < rows; r += 1024 / ORDER_CAND) {
        const double v = (double)proj[r * ORDER_CAND + k];
        a += v; b += v * v;
    }
    s1[t] = a; s2[t] = b;
    __syncthreads();
    for (u32 step = 512; step >= ORDER_CAND; step >>= 1) {       // threads t and t + step hold the same candidate
        if (t < step) { s1[t] += s1[t + step]; s2[t] += s2[t + step]; }
        __syncthreads();
    }
    if (t == 0) {
        u32 arg = 0;
        double top = -1.0;
        for (u32 c = 0; c < ncand; ++c) {
            const double n2 = (double)norm2[c];
            const double var = n2 > 0.0 ? (s2[c] - s1[c] * s1[c] / (double)rows) / n2 : 0.0;
            if (var > top) { top = var; arg = c; }
        }
        *best = arg;
        *pbar = (float)(s1[arg] / (double)rows);
    }
}

__global__ void __launch_bounds__(256) k_order_keys(const float* __restrict__ proj, u64 rows, const u32* __restrict__ best,
                                                    float* __restrict__ keys, u32* __restrict__ vals) {
    const u64 r = (u64)blockIdx.x * 256 + threadIdx.x;
    if (r >= rows) return;
    keys[r] = proj[r * ORDER_CAND + *best];
    vals[r] = (u32)r;
}

// One step of the power iteration towards the batch's direction of largest spread: v' = sum_i (p_i - pbar) q_i, the
// centred batch applied to its own projections (the sum of the weights is zero, so the mean of the batch drops out).
// k_order_back: partial sums over ORDER_CHUNKS row chunks, one column per thread, together with the column sums of
// the batch; k_order_finish: v' and the mean of the next projections, <mean row, v'>.
constexpr u32 ORDER_CHUNKS = 64;

__global__ void __launch_bounds__(256) k_order_back(const float* __restrict__ qrot, u64 rows, u32 d, const float* __restrict__ p,
                                                    const float* __restrict__ pbar, float* __restrict__ part_v,
                                                    float* __restrict__ part_m) {
    const u32 j = blockIdx.x * 256 + threadIdx.x;
    if (j >= d) return;
    const u64 per = (rows + ORDER_CHUNKS - 1) / ORDER_CHUNKS;
    const u64 r0 = (u64)blockIdx.y * per, r1 = r0 + per < rows ? r0 + per : rows;
    const float mean = *pbar;
    float av = 0.f, am = 0.f;
    for (u64 r = r0; r < r1; ++r) {
        const float x = qrot[r * d + j];
        av += (p[r] - mean) * x;
        am += x;
    }
    part_v[(u64)blockIdx.y * d + j] = av;
    part_m[(u64)blockIdx.y * d + j] = am;
}

__global__ void __launch_bounds__(1024) k_order_finish(const float* __restrict__ part_v, const float* __restrict__ part_m, u64 rows, u32 d,
                                                       float* __restrict__ v, float* __restrict__ pbar) {
    __shared__ double red[1024];
    double dot = 0.0;
    for (u32 j = threadIdx.x; j < d; j += 1024) {
        double a = 0.0, m = 0.0;
        for (u32 c = 0; c < ORDER_CHUNKS; ++c) { a += (double)part_v[(u64)c * d + j]; m += (double)part_m[(u64)c * d + j]; }
        v[j] = (float)a;
        dot += (double)(float)a * (m / (double)rows);
    }
    red[threadIdx.x] = dot;
    __syncthreads();
    for (u32 step = 512; step > 0; step >>= 1) {
        if (threadIdx.x < step) red[threadIdx.x] += red[threadIdx.x + step];
        __syncthreads();
    }
    if (threadIdx.x == 0) *pbar = (float)red[0];
}

// p[row] = <q_row, v>, one wave per row
__global__ void __launch_bounds__(64) k_order_project1(const float* __restrict__ qrot, u64 rows, u32 d, const float* __restrict__ v,
                                                       float* __restrict__ p) {
    const u64 row = blockIdx.x;
    if (row >= rows) return;
    float acc = 0.f;
    for (u32 c = threadIdx.x; c < d / 4; c += 64) {
        const float4 q = ((const float4*)(qrot + row * d))[c];
        const float4 x = ((const float4*)v)[c];
        acc += q.x * x.x + q.y * x.y + q.z * x.z + q.w * x.w;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
    if (threadIdx.x == 0) p[row] = acc;
}

}  // namespace

int pag_order_queries(pag_index* ix, const float* qrot, u64 nq, const u32** order) {
    *order = nullptr;
    const u32 ncand = std::min<u32>(ORDER_CAND, ix->n_entry);
    if (ncand == 0 || nq < 2 || nq >= (1ull << 31)) return PAG_OK;
    hipStream_t s = ix->stream;
    const u32 d = ix->L.d;
    size_t sort_bytes = 0;
    PAG_HIP(hipcub::DeviceRadixSort::SortPairs(nullptr, sort_bytes, (const float*)nullptr, (float*)nullptr, (const u32*)nullptr,
                                               (u32*)nullptr, (int)nq, 0, 32, s));
    // words: proj [nq * 16] | keys in [nq] | keys out [nq] | numbers [nq] | order [nq] | dirs [16 * d] | norm2 [16] |
    //        best, mean [16] | v [d] | partial sums [2 * 64 * d] | sort
    const u64 o_keys = nq * ORDER_CAND, o_keys2 = o_keys + nq, o_vals = o_keys2 + nq, o_order = o_vals + nq, o_dirs = o_order + nq;
    const u64 o_norm = o_dirs + (u64)ORDER_CAND * d, o_best = o_norm + ORDER_CAND, o_v = o_best + 16, o_part = o_v + d;
    const u64 o_sort = (o_part + 2ull * ORDER_CHUNKS * d + 63) / 64 * 64;   // 256-byte aligned
    const u64 need = o_sort + (sort_bytes + 3) / 4;
    if (ix->ws_order_cap < need) {
        if (ix->ws_order) (void)hipFree(ix->ws_order);
        ix->ws_order = nullptr; ix->ws_order_cap = 0;
        hipError_t e = hipMalloc((void**)&ix->ws_order, need * 4);
        if (e != hipSuccess) { pag_set_error(std::string("hipMalloc (query order): ") + hipGetErrorString(e)); return PAG_ENOMEM; }
        ix->ws_order_cap = need;
    }
    u32* w = ix->ws_order;
    float* proj = (float*)w;
    float* dirs = (float*)(w + o_dirs);
    float* norm2 = (float*)(w + o_norm);
    hipLaunchKernelGGL(k_order_dirs, dim3(ncand), dim3(64), 0, s, pag_vecs_of(ix), ix->entry, dirs, norm2);
    hipLaunchKernelGGL(k_order_project, dim3((unsigned)nq), dim3(64), 0, s, qrot, nq, d, dirs, ncand, proj);
    float* pbar = (float*)(w + o_best + 1);
    float* keys = (float*)(w + o_keys);
    float* v = (float*)(w + o_v);
    float* part_v = (float*)(w + o_part);
    float* part_m = part_v + (u64)ORDER_CHUNKS * d;
    hipLaunchKernelGGL(k_order_pick, dim3(1), dim3(1024), 0, s, proj, nq, ncand, norm2, w + o_best, pbar);
    hipLaunchKernelGGL(k_order_keys, dim3((unsigned)((nq + 255) / 256)), dim3(256), 0, s, proj, nq, w + o_best, keys, w + o_vals);
    // two steps from the best stored vector reach the direction of largest spread to within a percent of its variance
    for (int it = 0; it < 2; ++it) {
        hipLaunchKernelGGL(k_order_back, dim3((d + 255) / 256, ORDER_CHUNKS), dim3(256), 0, s, qrot, nq, d, keys, pbar, part_v, part_m);
        hipLaunchKernelGGL(k_order_finish, dim3(1), dim3(1024), 0, s, part_v, part_m, nq, d, v, pbar);
        hipLaunchKernelGGL(k_order_project1, dim3((unsigned)nq), dim3(64), 0, s, qrot, nq, d, v, keys);
    }
    PAG_HIP(hipGetLastError());
    PAG_HIP(hipcub::DeviceRadixSort::SortPairs((void*)(w + o_sort), sort_bytes, (const float*)(w + o_keys), (float*)(w + o_keys2),
                                               (const u32*)(w + o_vals), w + o_order, (int)nq, 0, 32, s));
    *order = w + o_order;
    return PAG_OK;
}

int pag_launch_rotate(hipStream_t s, const float* X, u64 rows, u32 d, const float* rot, float* out) {
    if (rows == 0) return PAG_OK;
    const u64 by = (rows + BM - 1) / BM;
    // gridDim.y is limited to 65535: walk the rows in slabs
    const u64 slab = 65535ull;
    for (u64 y0 = 0; y0 < by; y0 += slab) {
        const u64 ny = by - y0 < slab ? by - y0 : slab;
        const u64 r0 = y0 * BM;
        const u64 nrows = rows - r0 < ny * BM ? rows - r0 : ny * BM;
        dim3 grid((d + BN - 1) / BN, (unsigned)ny);
        hipLaunchKernelGGL(k_rotate, grid, dim3(256), 0, s, X + r0 * d, nrows, d, rot, out + r0 * d);
    }
    PAG_HIP(hipGetLastError());
    return PAG_OK;
}

int pag_launch_tables(hipStream_t s, const float* qrot, u64 rows, const pag_layout& L, const float* cb,
                      float* tables) {
    if (rows == 0) return PAG_OK;
    const u64 total = rows * L.Ppad * PAG_NCODE;
    hipLaunchKernelGGL(k_tables, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, qrot, rows, L.d, L.P,
                       L.Ppad, L.dsub, cb, tables);
    PAG_HIP(hipGetLastError());
    return PAG_OK;
}

int pag_launch_normalise(hipStream_t s, const float* X, u64 rows, u32 d, float* out) {
    if (rows == 0) return PAG_OK;
    hipLaunchKernelGGL(k_normalise, dim3((unsigned)rows), dim3(64), 0, s, X, rows, d, out);
    PAG_HIP(hipGetLastError());
    return PAG_OK;
}

int pag_launch_convert(hipStream_t s, const void* src, u32 src_half, void* dst, u32 dst_half, u64 count) {
    const u64 step = 1ull << 30;
    for (u64 o = 0; o < count; o += step) {
        const u64 c = count - o < step ? count - o : step;
        hipLaunchKernelGGL(k_convert, dim3((unsigned)((c + 255) / 256)), dim3(256), 0, s,
                           (const void*)((const char*)src + o * (src_half ? 2 : 4)), src_half,
                           (void*)((char*)dst + o * (dst_half ? 2 : 4)), dst_half, c);
    }
    PAG_HIP(hipGetLastError());
    return PAG_OK;
}

int pag_launch_zero_u32(hipStream_t s, u32* p, u64 count) {
    if (count == 0) return PAG_OK;
    hipLaunchKernelGGL(k_zero_u32, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, s, p, count);
    PAG_HIP(hipGetLastError());
    return PAG_OK;
}
