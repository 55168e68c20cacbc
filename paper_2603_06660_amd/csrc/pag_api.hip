// C ABI of the PAG library: argument checking, index life cycle, import / export, and the
// host side of pag_search (Alg. 2) -- everything that computes runs in the kernels.
#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <mutex>
#include <new>
#include <thread>
#include <vector>

#include "pag_internal.h"

static thread_local std::string g_last_error;
void pag_set_error(const std::string& msg) { g_last_error = msg; }
extern "C" const char* pag_last_error(void) { return g_last_error.c_str(); }

#define PAG_CHECK(cond, code, msg)                 \
    do {                                           \
        if (!(cond)) { pag_set_error(msg); return (code); } \
    } while (0)

// ---------------------------------------------------------------------------------------------
// Random structures of the method, drawn on the host once per index (Sec. 3.1; Alg. 1):
// the orthogonal transform Q from the Haar measure (Gaussian matrix, Gram-Schmidt with
// re-orthogonalisation) and, per subspace, independently rotated cross-polytopes.
// Counter-based generator: SplitMix64 on (seed, stream, counter) + Box-Muller.
// ---------------------------------------------------------------------------------------------
namespace {

struct Rng {
    uint64_t state;
    explicit Rng(uint64_t seed, uint64_t stream) : state(seed * 0x9E3779B97F4A7C15ull + stream * 0xD1B54A32D192ED03ull + 0x2545F4914F6CDD1Dull) {}
    uint64_t next() {
        uint64_t z = (state += 0x9E3779B97F4A7C15ull);
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    }
    double uniform() { return ((double)(next() >> 11) + 0.5) * (1.0 / 9007199254740992.0); }
    double normal() {
        const double u1 = uniform(), u2 = uniform();
        return std::sqrt(-2.0 * std::log(u1)) * std::cos(6.283185307179586476925 * u2);
    }
};

// Orthonormalise the columns of the dim x dim Gaussian matrix g (column-major) in place:
// classical Gram-Schmidt with one re-orthogonalisation pass, both inner loops split over threads.
void orthonormalise(std::vector<double>& g, uint32_t dim, unsigned threads) {
    std::vector<double> proj(dim);
    auto parallel = [&](uint32_t count, const std::function<void(uint32_t, uint32_t)>& fn) {
        if (threads <= 1 || count < 256) { fn(0, count); return; }
        std::vector<std::thread> th;
        for (unsigned t = 0; t < threads; ++t)
            th.emplace_back(fn, (uint32_t)((uint64_t)count * t / threads), (uint32_t)((uint64_t)count * (t + 1) / threads));
        for (auto& x : th) x.join();
    };
    for (uint32_t j = 0; j < dim; ++j) {
        double* aj = &g[(size_t)j * dim];
        for (int pass = 0; pass < 2 && j > 0; ++pass) {
            parallel(j, [&](uint32_t lo, uint32_t hi) {
                for (uint32_t i = lo; i < hi; ++i) {
                    const double* qi = &g[(size_t)i * dim];
                    double s = 0.0;
                    for (uint32_t k = 0; k < dim; ++k) s += qi[k] * aj[k];
                    proj[i] = s;
                }
            });
            parallel(j >= 256 ? dim : 0, [&](uint32_t lo, uint32_t hi) {
                for (uint32_t i = 0; i < j; ++i) {
                    const double* qi = &g[(size_t)i * dim];
                    const double p = proj[i];
                    for (uint32_t k = lo; k < hi; ++k) aj[k] -= p * qi[k];
                }
            });
            if (j < 256)
                for (uint32_t i = 0; i < j; ++i) {
                    const double* qi = &g[(size_t)i * dim];
                    const double p = proj[i];
                    for (uint32_t k = 0; k < dim; ++k) aj[k] -= p * qi[k];
                }
        }
        double nrm = 0.0;
        for (uint32_t k = 0; k < dim; ++k) nrm += aj[k] * aj[k];
        nrm = std::sqrt(nrm);
        for (uint32_t k = 0; k < dim; ++k) aj[k] /= nrm;
    }
}

void make_transform(uint32_t d, uint64_t seed, bool permutation, std::vector<float>& rot) {
    Rng rng(seed, 1);
    if (permutation) {
        // a signed permutation: row j has one entry +-1, in a column drawn by a Fisher-Yates shuffle
        std::vector<uint32_t> col(d);
        for (uint32_t j = 0; j < d; ++j) col[j] = j;
        for (uint32_t j = d - 1; j > 0; --j) std::swap(col[j], col[rng.next() % (j + 1)]);
        rot.assign((size_t)d * d, 0.f);
        for (uint32_t j = 0; j < d; ++j) rot[(size_t)j * d + col[j]] = (rng.next() & 1) ? 1.f : -1.f;
        return;
    }
    std::vector<double> g((size_t)d * d);
    for (auto& x : g) x = rng.normal();
    unsigned threads = std::max(1u, std::min(8u, std::thread::hardware_concurrency()));
    orthonormalise(g, d, threads);
    rot.resize((size_t)d * d);
    // orthonormal columns are as good as rows: rot[j][k] = column j, element k
    for (size_t i = 0; i < rot.size(); ++i) rot[i] = (float)g[i];
}

// cb[l][j][k]: per subspace, cross-polytopes rotated independently; from each polytope its axes in
// order, first with sign +, then with sign -, until 16 vectors are collected; norm 1/sqrt(P).
void make_codebooks(uint32_t d, uint32_t P, uint64_t seed, std::vector<float>& cb) {
    const uint32_t ds = d / P;
    Rng rng(seed, 2);
    cb.assign((size_t)P * PAG_NCODE * ds, 0.f);
    const double scale = 1.0 / std::sqrt((double)P);
    std::vector<double> g((size_t)ds * ds);
    for (uint32_t l = 0; l < P; ++l) {
        uint32_t j = 0;
        while (j < PAG_NCODE) {
            for (auto& x : g) x = rng.normal();
            orthonormalise(g, ds, 1);
            const uint32_t k = std::min<uint32_t>(ds, (PAG_NCODE - j) / 2);
            for (uint32_t a = 0; a < k; ++a)
                for (uint32_t e = 0; e < ds; ++e) {
                    const double v = g[(size_t)a * ds + e] * scale;
                    cb[((size_t)l * PAG_NCODE + j + a) * ds + e] = (float)v;
                    cb[((size_t)l * PAG_NCODE + j + k + a) * ds + e] = (float)(-v);
                }
            j += 2 * k;
        }
    }
}

int make_layout(uint32_t d, uint32_t P, uint32_t deg, pag_layout* L) {
    PAG_CHECK(d > 0 && P > 0 && deg > 0, PAG_EINVAL, "d, num_subspaces and max_degree must be positive");
    PAG_CHECK(d % P == 0, PAG_EINVAL, "d must be divisible by num_subspaces");
    PAG_CHECK(d % 4 == 0 && d <= 3072, PAG_EUNSUPPORTED, "this build needs d % 4 == 0 and d <= 3072");
    PAG_CHECK(P <= 8 * PAG_MAX_CW, PAG_EUNSUPPORTED, "this build needs num_subspaces <= 64");
    PAG_CHECK(deg <= PAG_MAX_DEG, PAG_EUNSUPPORTED, "this build needs max_degree <= 64");
    L->d = d; L->P = P; L->dsub = d / P; L->deg = deg;
    L->Ppad = P <= 16 ? 16 : (P <= 32 ? 32 : 64);
    L->cw = L->Ppad / 8;
    L->off_a = deg * 4;
    L->off_c = deg * 8;
    L->off_codes = (deg * 12 + 15) / 16 * 16;
    L->rec_bytes = (L->off_codes + deg * L->cw * 4 + 127) / 128 * 128;
    return PAG_OK;
}

int check_params(const pag_params* p) {
    PAG_CHECK(p != nullptr, PAG_EINVAL, "params is null");
    PAG_CHECK(p->struct_size == sizeof(pag_params), PAG_EINVAL, "pag_params.struct_size does not match this library");
    PAG_CHECK(p->metric >= PAG_L2 && p->metric <= PAG_COS, PAG_EINVAL, "unknown metric");
    PAG_CHECK(p->ef_construction >= 1, PAG_EINVAL, "ef_construction must be >= 1");
    PAG_CHECK(p->search_b <= PAG_MAX_B, PAG_EUNSUPPORTED, "search_b above 1024 is not built");
    // the reverse-edge pairs of one batch (2 * max_degree per vector) are counted in 32 bits
    PAG_CHECK(p->insert_subbatch <= (1u << 20), PAG_EUNSUPPORTED, "insert_subbatch above 2^20 is not built");
    return PAG_OK;
}

// Runs the body of an entry point; no exception leaves the library (host allocations can throw).
template <typename F>
int guarded(const char* what, F&& body) {
    try {
        return body();
    } catch (const std::bad_alloc&) {
        pag_set_error(std::string(what) + ": host allocation failed");
        return PAG_ENOMEM;
    } catch (const std::exception& e) {
        pag_set_error(std::string(what) + ": " + e.what());
        return PAG_EINVAL;
    }
}

template <typename T>
int dev_alloc(T** p, u64 count) {
    *p = nullptr;
    if (count == 0) count = 1;
    hipError_t e = hipMalloc((void**)p, count * sizeof(T));
    if (e != hipSuccess) { pag_set_error(std::string("hipMalloc: ") + hipGetErrorString(e)); return PAG_ENOMEM; }
    return PAG_OK;
}

template <typename T>
int ensure_ws(T** p, u64* cap, u64 need) {
    if (*cap >= need) return PAG_OK;
    if (*p) { hipError_t e = hipFree(*p); (void)e; *p = nullptr; *cap = 0; }
    int rc = dev_alloc(p, need);
    if (rc == PAG_OK) *cap = need;
    return rc;
}

struct DeviceGuard {
    int prev = -1;
    explicit DeviceGuard(int dev) { if (hipGetDevice(&prev) != hipSuccess) prev = -1; if (prev != dev) (void)hipSetDevice(dev); else prev = -1; }
    ~DeviceGuard() { if (prev >= 0) (void)hipSetDevice(prev); }
};

}  // namespace

// The workspace of pag_search_static: one file-scope device array.  Each GPU the library runs on holds its own copy,
// at its own address, until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress: the device address is looked up once per device, with that device current, and used from
// then on.
static __device__ __align__(256) unsigned char scratch[PAG_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
unsigned char* g_scratch_ptr[kMaxDevices];        // device address of `scratch` per device, null until looked up

int scratch_of(int device, unsigned char** out) {
    PAG_CHECK(device >= 0 && device < kMaxDevices, PAG_EUNSUPPORTED, "pag_search_static: device number above 63");
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* p = nullptr;
        PAG_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));      // the current device's copy
        PAG_CHECK(p != nullptr, PAG_EHIP, "pag_search_static: the scratch array has no device address");
        g_scratch_ptr[device] = (unsigned char*)p;
    }
    *out = g_scratch_ptr[device];
    return PAG_OK;
}
}  // namespace

namespace {

// allocate the HBM-resident parts of an index for `capacity` nodes
int alloc_index(pag_index* ix) {
    int rc;
    {
        uint8_t* raw = nullptr;
        if ((rc = dev_alloc(&raw, ix->capacity * ix->L.d * pag_vec_elem(ix)))) return rc;
        ix->vec = raw;
    }
    if ((rc = dev_alloc(&ix->rec, ix->capacity * ix->L.rec_bytes))) return rc;
    if ((rc = dev_alloc(&ix->e2, ix->capacity * ix->L.deg))) return rc;
    if ((rc = dev_alloc(&ix->rot, (u64)ix->L.d * ix->L.d))) return rc;
    if ((rc = dev_alloc(&ix->cb, (u64)ix->L.P * PAG_NCODE * ix->L.dsub))) return rc;
    if ((rc = dev_alloc(&ix->entry, 1024))) return rc;
    if ((rc = dev_alloc(&ix->d_qcounter, 4))) return rc;
    if ((rc = dev_alloc(&ix->d_counters, CTR_COUNT))) return rc;
    PAG_HIP(hipMemsetAsync(ix->d_counters, 0, CTR_COUNT * sizeof(u64), ix->stream));
    for (auto& e : ix->ev) PAG_HIP(hipEventCreate(&e));
    // pag_search_static must find its workspace without loading or allocating anything: look it up now
    unsigned char* static_ws = nullptr;
    return scratch_of(ix->device, &static_ws);
}

pag_index* new_index(const pag_params* p, uint32_t d) {
    pag_index* ix = new pag_index();
    std::memset((void*)ix, 0, sizeof(*ix));
    (void)hipGetDevice(&ix->device);
    ix->stream = (hipStream_t)p->stream;
    ix->metric = p->metric;
    ix->efC = p->ef_construction;
    ix->search_b = p->search_b;
    ix->subbatch = p->insert_subbatch;
    ix->flags = p->flags & ~PAG_FLAG_FP16_VECTORS;
    ix->vec_half = (p->flags & PAG_FLAG_FP16_VECTORS) ? 1u : 0u;
    ix->seed = p->seed;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, ix->device) == hipSuccess) ix->num_cu = prop.multiProcessorCount;
    if (ix->num_cu <= 0) ix->num_cu = 256;
    (void)d;
    return ix;
}

// normalise (COS) + rotate `rows` raw vectors X (dev) into rows [row0, row0 + rows) of the store
int ingest(pag_index* ix, const float* X, u64 rows, u64 row0) {
    const u32 d = ix->L.d;
    int rc;
    const u64 slab = 1ull << 18;
    for (u64 s0 = 0; s0 < rows; s0 += slab) {
        const u64 cnt = std::min<u64>(slab, rows - s0);
        const float* src = X + s0 * d;
        if (ix->metric == PAG_COS) {
            if ((rc = ensure_ws(&ix->ws_norm, &ix->ws_norm_cap, cnt * d))) return rc;
            if ((rc = pag_launch_normalise(ix->stream, src, cnt, d, ix->ws_norm))) return rc;
            src = ix->ws_norm;
        }
        if (!ix->vec_half) {
            if ((rc = pag_launch_rotate(ix->stream, src, cnt, d, ix->rot, (float*)ix->vec + (row0 + s0) * d))) return rc;
        } else {
            // fp32 result of the rotation first, then one rounding to the 16-bit store
            if ((rc = ensure_ws(&ix->ws_qrot, &ix->ws_qrot_cap, cnt * d))) return rc;
            if ((rc = pag_launch_rotate(ix->stream, src, cnt, d, ix->rot, ix->ws_qrot))) return rc;
            if ((rc = pag_launch_convert(ix->stream, ix->ws_qrot, 0, (__half*)ix->vec + (row0 + s0) * d, 1, cnt * d))) return rc;
        }
    }
    return PAG_OK;
}

}  // namespace

// ---------------------------------------------------------------------------------------------

extern "C" int pag_free(pag_index* ix) {
    if (!ix) return PAG_OK;
    DeviceGuard g(ix->device);
    (void)hipStreamSynchronize(ix->stream);
    void* ptrs[] = { ix->vec, ix->rec, ix->e2, ix->rot, ix->cb, ix->entry, ix->ws_qrot, ix->ws_tab, ix->ws_norm,
                     ix->ws_bitmap, ix->ws_rings, ix->ws_order, ix->d_qcounter, ix->d_counters };
    for (void* p : ptrs) if (p) (void)hipFree(p);
    for (auto& e : ix->ev) if (e) (void)hipEventDestroy(e);
    delete ix;
    return PAG_OK;
}

extern "C" int pag_build(const float* D, uint64_t n, uint32_t d, const pag_params* params, pag_index** out) {
    PAG_CHECK(out != nullptr, PAG_EINVAL, "out is null");
    *out = nullptr;
    int rc = check_params(params);
    if (rc) return rc;
    PAG_CHECK(D != nullptr && n > 0, PAG_EINVAL, "D is null or n == 0");
    PAG_CHECK(n < (1ull << 31), PAG_EUNSUPPORTED, "n must be below 2^31");
    pag_layout L;
    if ((rc = make_layout(d, params->num_subspaces, params->max_degree, &L))) return rc;
    PAG_CHECK(!(params->flags & PAG_FLAG_FP16_VECTORS) || d % 8 == 0, PAG_EUNSUPPORTED,
              "PAG_FLAG_FP16_VECTORS needs d % 8 == 0");
    pag_index* ix = nullptr;
    rc = guarded("pag_build", [&]() -> int {
        int rc;
        ix = new_index(params, d);
        ix->L = L;
        ix->capacity = std::max<u64>(params->capacity, n);
        if (ix->capacity >= (1ull << 31)) { pag_set_error("capacity must be below 2^31"); return PAG_EUNSUPPORTED; }
        const auto t0 = std::chrono::steady_clock::now();
        if ((rc = alloc_index(ix))) return rc;
        std::vector<float> rot, cb;
        make_transform(d, params->seed, (params->flags & PAG_FLAG_PERMUTATION_TRANSFORM) != 0, rot);
        make_codebooks(d, L.P, params->seed, cb);
        hipError_t e = hipMemcpyAsync(ix->rot, rot.data(), rot.size() * 4, hipMemcpyHostToDevice, ix->stream);
        if (e == hipSuccess) e = hipMemcpyAsync(ix->cb, cb.data(), cb.size() * 4, hipMemcpyHostToDevice, ix->stream);
        if (e == hipSuccess) e = hipMemsetAsync(ix->rec, 0xFF, ix->capacity * L.rec_bytes, ix->stream);
        if (e == hipSuccess) e = hipStreamSynchronize(ix->stream);
        if (e != hipSuccess) { pag_set_error(std::string("pag_build upload: ") + hipGetErrorString(e)); return PAG_EHIP; }
        if ((rc = ingest(ix, D, n, 0))) return rc;
        ix->n = 0;
        if ((rc = pag_build_range(ix, 0, n))) return rc;
        ix->n = n;
        ix->last_build_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
        return PAG_OK;
    });
    if (rc) { pag_free(ix); return rc; }
    *out = ix;
    return PAG_OK;
}

extern "C" int pag_insert(pag_index* ix, const float* X, uint64_t m) {
    PAG_CHECK(ix != nullptr, PAG_EINVAL, "index is null");
    if (m == 0) return PAG_OK;
    PAG_CHECK(X != nullptr, PAG_EINVAL, "X is null");
    PAG_CHECK(ix->n + m <= ix->capacity, PAG_ECAPACITY, "pag_insert: capacity exceeded");
    PAG_CHECK(!ix->insert_failed, PAG_EINVAL, "pag_insert: an earlier pag_insert on this index failed half way; it takes no more vectors");
    DeviceGuard g(ix->device);
    const auto t0 = std::chrono::steady_clock::now();
    const u32 entry_before = ix->n_entry;
    int rc = guarded("pag_insert", [&]() -> int {
        int rc;
        if ((rc = ingest(ix, X, m, ix->n))) return rc;
        return pag_build_range(ix, ix->n, ix->n + m);
    });
    if (rc) {
        // searches go on over the n published nodes (ids >= n are ignored); the entry list is theirs again
        ix->n_entry = entry_before;
        ix->insert_failed = 1;
        return rc;
    }
    // publish: every kernel of the insertion has finished (pag_build_range synchronises), searchers may now see the nodes
    __atomic_store_n(&ix->n, ix->n + m, __ATOMIC_RELEASE);
    ix->last_build_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
    return PAG_OK;
}

extern "C" int pag_describe(const pag_index* ix, pag_arrays* out) {
    PAG_CHECK(ix && out, PAG_EINVAL, "null argument");
    PAG_CHECK(out->struct_size == sizeof(pag_arrays), PAG_EINVAL, "pag_arrays.struct_size does not match this library");
    out->metric = ix->metric; out->n = ix->n; out->d = ix->L.d; out->num_subspaces = ix->L.P;
    out->max_degree = ix->L.deg; out->n_entry = ix->n_entry;
    return PAG_OK;
}

static int export_impl(const pag_index* ix, pag_arrays* out) {
    PAG_CHECK(ix && out, PAG_EINVAL, "null argument");
    PAG_CHECK(out->struct_size == sizeof(pag_arrays), PAG_EINVAL, "pag_arrays.struct_size does not match this library");
    PAG_CHECK(out->vectors && out->adj && out->a && out->c && out->e2 && out->codes && out->rotation &&
              out->codebooks && out->entry, PAG_EINVAL, "pag_export: every output array must be allocated");
    DeviceGuard g(ix->device);
    const pag_layout& L = ix->L;
    const u64 n = ix->n;
    PAG_HIP(hipStreamSynchronize(ix->stream));
    if (!ix->vec_half) {
        PAG_HIP(hipMemcpy(out->vectors, ix->vec, n * L.d * 4, hipMemcpyDeviceToHost));
    } else {
        const u64 vslab = 1ull << 18;
        float* tmp = nullptr;
        int rc2 = dev_alloc(&tmp, std::min<u64>(vslab, n) * L.d);
        if (rc2) return rc2;
        for (u64 s0 = 0; s0 < n; s0 += vslab) {
            const u64 cnt = std::min<u64>(vslab, n - s0);
            rc2 = pag_launch_convert(ix->stream, (const __half*)ix->vec + s0 * L.d, 1, tmp, 0, cnt * L.d);
            hipError_t e2 = rc2 ? hipSuccess : hipStreamSynchronize(ix->stream);
            if (!rc2 && e2 == hipSuccess) e2 = hipMemcpy(out->vectors + s0 * L.d, tmp, cnt * L.d * 4, hipMemcpyDeviceToHost);
            if (rc2 || e2 != hipSuccess) {
                (void)hipFree(tmp);
                if (!rc2) { pag_set_error(std::string("pag_export: ") + hipGetErrorString(e2)); return PAG_EHIP; }
                return rc2;
            }
        }
        (void)hipFree(tmp);
    }
    PAG_HIP(hipMemcpy(out->e2, ix->e2, n * L.deg * 4, hipMemcpyDeviceToHost));
    PAG_HIP(hipMemcpy(out->rotation, ix->rot, (u64)L.d * L.d * 4, hipMemcpyDeviceToHost));
    PAG_HIP(hipMemcpy(out->codebooks, ix->cb, (u64)L.P * PAG_NCODE * L.dsub * 4, hipMemcpyDeviceToHost));
    PAG_HIP(hipMemcpy(out->entry, ix->entry, ix->n_entry * 4, hipMemcpyDeviceToHost));
    const u64 slab = 1 << 16;
    std::vector<uint8_t> buf(std::min<u64>(slab, std::max<u64>(n, 1)) * L.rec_bytes);
    for (u64 s = 0; s < n; s += slab) {
        const u64 cnt = std::min<u64>(slab, n - s);
        PAG_HIP(hipMemcpy(buf.data(), ix->rec + s * L.rec_bytes, cnt * L.rec_bytes, hipMemcpyDeviceToHost));
        for (u64 i = 0; i < cnt; ++i) {
            const uint8_t* rec = buf.data() + i * L.rec_bytes;
            const u64 o = (s + i) * L.deg;
            std::memcpy(out->adj + o, rec, L.deg * 4);
            std::memcpy(out->a + o, rec + L.off_a, L.deg * 4);
            std::memcpy(out->c + o, rec + L.off_c, L.deg * 4);
            const u32* cw = (const u32*)(rec + L.off_codes);
            for (u32 e = 0; e < L.deg; ++e)
                for (u32 l = 0; l < L.P; ++l)
                    out->codes[(o + e) * L.P + l] = (uint8_t)((cw[e * L.cw + l / 8] >> (4 * (l % 8))) & 15u);
        }
    }
    out->metric = ix->metric; out->n = n; out->d = L.d; out->num_subspaces = L.P; out->max_degree = L.deg;
    out->n_entry = ix->n_entry;
    return PAG_OK;
}

extern "C" int pag_export(const pag_index* ix, pag_arrays* out) {
    return guarded("pag_export", [&]() { return export_impl(ix, out); });
}

static int import_impl(const pag_arrays* in, const pag_params* params, pag_index** out) {
    PAG_CHECK(out != nullptr, PAG_EINVAL, "out is null");
    *out = nullptr;
    int rc = check_params(params);
    if (rc) return rc;
    PAG_CHECK(in != nullptr && in->struct_size == sizeof(pag_arrays), PAG_EINVAL, "pag_arrays is null or of another size");
    PAG_CHECK(in->vectors && in->adj && in->a && in->c && in->e2 && in->codes && in->rotation && in->codebooks &&
              in->entry, PAG_EINVAL, "pag_import: every array is required");
    PAG_CHECK(in->n > 0 && in->n < (1ull << 31), PAG_EINVAL, "pag_import: n out of range");
    PAG_CHECK(in->n_entry >= 1 && in->n_entry <= 1024, PAG_EINVAL, "pag_import: n_entry must be in 1..1024");
    PAG_CHECK(in->metric >= PAG_L2 && in->metric <= PAG_COS, PAG_EINVAL, "pag_import: unknown metric");
    pag_layout L;
    if ((rc = make_layout(in->d, in->num_subspaces, in->max_degree, &L))) return rc;
    const u64 n = in->n;
    for (u64 i = 0; i < n * L.deg; ++i)
        PAG_CHECK(in->adj[i] == PAG_EMPTY || in->adj[i] < n, PAG_EINVAL, "pag_import: neighbour id out of range");
    // the search admits the unseen neighbours of a node together and relies on their keys being
    // distinct: a node may not list a neighbour twice, nor the entry list a node twice
    for (u64 u = 0; u < n; ++u) {
        const u32* row = in->adj + u * L.deg;
        for (u32 i = 1; i < L.deg; ++i)
            for (u32 j = 0; j < i; ++j)
                PAG_CHECK(row[i] == PAG_EMPTY || row[i] != row[j], PAG_EINVAL, "pag_import: a node lists a neighbour twice");
    }
    for (u32 i = 0; i < in->n_entry; ++i) {
        PAG_CHECK(in->entry[i] < n, PAG_EINVAL, "pag_import: entry id out of range");
        for (u32 j = 0; j < i; ++j) PAG_CHECK(in->entry[i] != in->entry[j], PAG_EINVAL, "pag_import: entry id listed twice");
    }
    for (u64 i = 0; i < n * L.deg * L.P; ++i) PAG_CHECK(in->codes[i] < PAG_NCODE, PAG_EINVAL, "pag_import: code above 15");
    PAG_CHECK(!(params->flags & PAG_FLAG_FP16_VECTORS) || in->d % 8 == 0, PAG_EUNSUPPORTED,
              "PAG_FLAG_FP16_VECTORS needs d % 8 == 0");
    // host staging first: nothing below this point allocates host memory
    const u64 slab = 1 << 16;
    std::vector<uint8_t> buf(std::min<u64>(slab, n) * L.rec_bytes);
    pag_index* ix = new_index(params, in->d);
    ix->metric = in->metric;
    ix->L = L;
    ix->capacity = std::max<u64>(params->capacity, n);
    if ((rc = alloc_index(ix))) { pag_free(ix); return rc; }
    auto fail = [&](hipError_t e) { pag_set_error(std::string("pag_import: ") + hipGetErrorString(e)); pag_free(ix); return PAG_EHIP; };
    hipError_t e;
    if ((e = hipMemsetAsync(ix->rec, 0xFF, ix->capacity * L.rec_bytes, ix->stream)) != hipSuccess) return fail(e);
    if ((e = hipStreamSynchronize(ix->stream)) != hipSuccess) return fail(e);
    if (!ix->vec_half) {
        if ((e = hipMemcpy(ix->vec, in->vectors, n * L.d * 4, hipMemcpyHostToDevice)) != hipSuccess) return fail(e);
    } else {
        const u64 vslab = 1ull << 18;
        if ((rc = ensure_ws(&ix->ws_qrot, &ix->ws_qrot_cap, std::min<u64>(vslab, n) * L.d))) { pag_free(ix); return rc; }
        for (u64 s0 = 0; s0 < n; s0 += vslab) {
            const u64 cnt = std::min<u64>(vslab, n - s0);
            if ((e = hipMemcpy(ix->ws_qrot, in->vectors + s0 * L.d, cnt * L.d * 4, hipMemcpyHostToDevice)) != hipSuccess) return fail(e);
            if ((rc = pag_launch_convert(ix->stream, ix->ws_qrot, 0, (__half*)ix->vec + s0 * L.d, 1, cnt * L.d))) { pag_free(ix); return rc; }
            if ((e = hipStreamSynchronize(ix->stream)) != hipSuccess) return fail(e);
        }
    }
    if ((e = hipMemcpy(ix->e2, in->e2, n * L.deg * 4, hipMemcpyHostToDevice)) != hipSuccess) return fail(e);
    if ((e = hipMemcpy(ix->rot, in->rotation, (u64)L.d * L.d * 4, hipMemcpyHostToDevice)) != hipSuccess) return fail(e);
    if ((e = hipMemcpy(ix->cb, in->codebooks, (u64)L.P * PAG_NCODE * L.dsub * 4, hipMemcpyHostToDevice)) != hipSuccess) return fail(e);
    if ((e = hipMemcpy(ix->entry, in->entry, in->n_entry * 4, hipMemcpyHostToDevice)) != hipSuccess) return fail(e);
    ix->n_entry = in->n_entry;
    for (u64 s = 0; s < n; s += slab) {
        const u64 cnt = std::min<u64>(slab, n - s);
        std::memset(buf.data(), 0, cnt * L.rec_bytes);
        for (u64 i = 0; i < cnt; ++i) {
            uint8_t* rec = buf.data() + i * L.rec_bytes;
            const u64 o = (s + i) * L.deg;
            std::memcpy(rec, in->adj + o, L.deg * 4);
            std::memcpy(rec + L.off_a, in->a + o, L.deg * 4);
            std::memcpy(rec + L.off_c, in->c + o, L.deg * 4);
            u32* cw = (u32*)(rec + L.off_codes);
            for (u32 ed = 0; ed < L.deg; ++ed)
                for (u32 l = 0; l < L.P; ++l)
                    cw[ed * L.cw + l / 8] |= (u32)(in->codes[(o + ed) * L.P + l] & 15u) << (4 * (l % 8));
        }
        if ((e = hipMemcpy(ix->rec + s * L.rec_bytes, buf.data(), cnt * L.rec_bytes, hipMemcpyHostToDevice)) != hipSuccess) return fail(e);
    }
    ix->n = n;
    *out = ix;
    return PAG_OK;
}

extern "C" int pag_import(const pag_arrays* in, const pag_params* params, pag_index** out) {
    if (out) *out = nullptr;
    return guarded("pag_import", [&]() { return import_impl(in, params, out); });
}

extern "C" int pag_get_counters(const pag_index* ix, pag_counters* out) {
    PAG_CHECK(ix && out, PAG_EINVAL, "null argument");
    PAG_CHECK(out->struct_size == sizeof(pag_counters), PAG_EINVAL, "pag_counters.struct_size does not match this library");
    DeviceGuard g(ix->device);
    u64 h[CTR_COUNT];
    PAG_HIP(hipStreamSynchronize(ix->stream));
    PAG_HIP(hipMemcpy(h, ix->d_counters, sizeof h, hipMemcpyDeviceToHost));
    out->adj_record_bytes = ix->L.rec_bytes;
    out->queries = h[CTR_QUERIES]; out->hops = h[CTR_HOPS]; out->tests = h[CTR_TESTS]; out->passes = h[CTR_PASSES];
    out->exact = h[CTR_EXACT]; out->rounds = h[CTR_ROUNDS]; out->rf_overflow = h[CTR_RF_OVER];
    out->rt_overflow = h[CTR_RT_OVER]; out->seen_spills = h[CTR_SPILLS];
    out->last_search_kernel_ms = ix->last_search_ms;
    out->last_prepare_ms = ix->last_prepare_ms;
    out->last_build_ms = ix->last_build_ms;
    for (int i = 0; i < 6; ++i) out->phase_cycles[i] = h[CTR_PHASE0 + i];
    out->relinked_batches = ix->relinked_batches;
    for (int i = 0; i < 4; ++i) out->last_build_phase_ms[i] = ix->build_phase_ms[i];
    return PAG_OK;
}

extern "C" int pag_reset_counters(pag_index* ix) {
    PAG_CHECK(ix, PAG_EINVAL, "null argument");
    DeviceGuard g(ix->device);
    int rc = pag_launch_zero_u32(ix->stream, (u32*)ix->d_counters, CTR_COUNT * 2);
    if (rc) return rc;
    PAG_HIP(hipStreamSynchronize(ix->stream));
    return PAG_OK;
}

extern "C" int pag_set_search_options(pag_index* ix, uint32_t search_b, uint32_t flags) {
    PAG_CHECK(ix, PAG_EINVAL, "null argument");
    PAG_CHECK(search_b <= PAG_MAX_B, PAG_EUNSUPPORTED, "search_b above 1024 is not built");
    ix->search_b = search_b;
    const u32 search_bits = PAG_FLAG_NO_PRT | PAG_FLAG_EXACT_TEST_COUNT | PAG_FLAG_KEEP_QUERY_ORDER;
    ix->flags = (ix->flags & ~search_bits) | (flags & search_bits);           // index-time bits stay as built
    return PAG_OK;
}

extern "C" int pag_set_seen_capacity_log2(pag_index* ix, uint32_t log2_slots) {
    PAG_CHECK(ix, PAG_EINVAL, "null argument");
    PAG_CHECK(log2_slots == 0 || (log2_slots >= 6 && log2_slots <= 13), PAG_EINVAL, "seen capacity log2 must be 0 or in 6..13");
    ix->seen_log2 = log2_slots;
    return PAG_OK;
}

// ---------------------------------------------------------------------------------------------
// search
// ---------------------------------------------------------------------------------------------

// normalisation (COS, into `norm`), rotation and projection tables of nq queries; allocates nothing
static int prepare_into(const pag_index* ix, const float* Q, u64 nq, float* norm, float* qrot, float* tables) {
    const float* src = Q;
    int rc;
    if (ix->metric == PAG_COS) {
        if ((rc = pag_launch_normalise(ix->stream, Q, nq, ix->L.d, norm))) return rc;
        src = norm;
    }
    if ((rc = pag_launch_rotate(ix->stream, src, nq, ix->L.d, ix->rot, qrot))) return rc;
    return pag_launch_tables(ix->stream, qrot, nq, ix->L, ix->cb, tables);
}

static int prepare(pag_index* ix, const float* Q, u64 nq, float* qrot, float* tables) {
    int rc;
    if (ix->metric == PAG_COS && (rc = ensure_ws(&ix->ws_norm, &ix->ws_norm_cap, nq * ix->L.d))) return rc;
    return prepare_into(ix, Q, nq, ix->ws_norm, qrot, tables);
}

// Seen-set sizing.  A search expected to compute at most ~1000 exact distances (entries + a few per
// visited node) gets an exact LDS hash that holds all of them.  Longer searches keep every id in the
// per-wave HBM bitmap, guarded by a 4 KB LDS Bloom filter, and use a small LDS table as a cache of
// recently admitted ids: large LDS tables cost more in occupancy than the bitmap costs in loads.
static void seen_sizes_for(const pag_index* ix, u32 ef, u32 b, u32* hlog, u32* blog) {
    const u32 expected = b + 8 * std::max(ef, b);
    if (expected <= 1024) {
        u32 lg = 9;
        while ((1u << lg) < 2 * expected && lg < 11) ++lg;
        *hlog = lg; *blog = 0;
    } else {
        *hlog = 9; *blog = 15;
    }
    if (ix->seen_log2) *hlog = ix->seen_log2;
}

// Plans a search: fills the part of SearchArgs that depends only on the index and (b, ef), the LDS carve-up and the
// largest useful grid.  Allocates nothing.
static int search_plan(const pag_index* ix, u32 b, u32 ef, u64 n_limit, SearchArgs* a, u32* lds, int* grid) {
    const pag_layout& L = ix->L;
    std::memset((void*)a, 0, sizeof(*a));
    a->vec = ix->vec; a->rec = ix->rec; a->entry = ix->entry;
    a->n_entry = (u32)std::min<u64>(ix->n_entry, n_limit);
    a->n_limit = (u32)n_limit;
    a->d = L.d; a->deg = L.deg; a->Ppad = L.Ppad; a->cw = L.cw; a->rec_bytes = L.rec_bytes;
    a->off_a = L.off_a; a->off_c = L.off_c; a->off_codes = L.off_codes;
    a->b = b; a->Rmax = std::max<u32>(1, (ef + b - 1) / b);
    seen_sizes_for(ix, ef, b, &a->hlog, &a->blog);
    a->flags = ix->flags;
    a->qcounter = ix->d_qcounter; a->counters = ix->d_counters;
    *lds = (u32)pag_search_lds_bytes(L, b, a->hlog, a->blog, a);
    if (*lds > 65536) { pag_set_error("search: working set, tables and seen set need more than 64 KB of LDS per wave"); return PAG_EUNSUPPORTED; }
    int rc = pag_search_max_grid(ix, b, *lds, grid);
    if (rc) return rc;
    // Long searches use the LDS hash only for their first nodes.  Where the registers of the kernel
    // would allow more waves per CU than this LDS footprint does, a smaller hash buys them.  The
    // comparison is made with half a KB of slack: a footprint that only just fits the count the
    // occupancy query reports did not reach it in measurements.
    if (a->blog && !ix->seen_log2) {
        const u32 slack = 512;
        int best = 0;
        if ((rc = pag_search_max_grid(ix, b, *lds + slack, &best))) return rc;
        for (u32 lg = a->hlog - 1; lg >= 7; --lg) {
            SearchArgs t = *a;
            t.hlog = lg;
            const u32 l2 = (u32)pag_search_lds_bytes(L, b, lg, t.blog, &t);
            int g2 = 0;
            if ((rc = pag_search_max_grid(ix, b, l2 + slack, &g2))) return rc;
            if (g2 > best) {
                best = g2;
                *a = t; *lds = l2;
                if ((rc = pag_search_max_grid(ix, b, l2, grid))) return rc;
            }
        }
    }
    // per-wave spill bitmaps of the seen set: one bit per node, rounded to 16 bytes
    a->bitmap_words = ((u64)ix->capacity + 127) / 128 * 4;
    return PAG_OK;
}

// The plan plus the workspaces it needs (grown on demand); shared with indexing.
int pag_search_common(pag_index* ix, u32 b, u32 ef, u64 n_limit, SearchArgs* a, u32* lds, int* grid) {
    int rc = search_plan(ix, b, ef, n_limit, a, lds, grid);
    if (rc) return rc;
    const u64 need = (u64)*grid * a->bitmap_words;
    if (ix->ws_bitmap_cap < need) {
        // a fresh buffer starts dirty: clear it once; every wave leaves its slice clean afterwards
        if ((rc = ensure_ws(&ix->ws_bitmap, &ix->ws_bitmap_cap, need))) return rc;
        PAG_HIP(hipMemsetAsync(ix->ws_bitmap, 0, need * 4, ix->stream));
    }
    a->bitmap = ix->ws_bitmap;
    if (b > PAG_LDS_RING_MAX_B) {
        if ((rc = ensure_ws(&ix->ws_rings, &ix->ws_rings_cap, (u64)*grid * 3 * (u64)(a->ring_mask + 1)))) return rc;
        a->rings = ix->ws_rings;
    }
    return PAG_OK;
}

// The search of one batch with the workspaces, counters, events and stream of `ix` (an index, or a
// searcher's view of one).
static int search_impl(pag_index* ix, const float* Q, uint64_t nq, uint32_t K, uint32_t efS, int64_t* ids,
                       float* dists) {
    if (nq == 0) return PAG_OK;
    PAG_CHECK(Q && ids && dists, PAG_EINVAL, "Q, ids or dists is null");
    PAG_CHECK(K >= 1 && K <= ix->n, PAG_EINVAL, "K must be in 1..n");
    PAG_CHECK(efS >= 1, PAG_EINVAL, "efS must be >= 1");
    PAG_CHECK(nq < (1ull << 31), PAG_EINVAL, "nq must be below 2^31");
    const u32 b = ix->search_b ? ix->search_b : std::max<u32>(10, K);
    PAG_CHECK(b >= K, PAG_EINVAL, "search_b must be >= K");
    PAG_CHECK(b <= PAG_MAX_B, PAG_EUNSUPPORTED, "working sets above 1024 nodes (K > 1024) are not built");
    DeviceGuard g(ix->device);
    const pag_layout& L = ix->L;
    int rc;
    if ((rc = ensure_ws(&ix->ws_qrot, &ix->ws_qrot_cap, nq * L.d))) return rc;
    if ((rc = ensure_ws(&ix->ws_tab, &ix->ws_tab_cap, nq * L.Ppad * PAG_NCODE))) return rc;
    SearchArgs a;
    u32 lds = 0;
    int grid = 0;
    if ((rc = pag_search_common(ix, b, efS, ix->n, &a, &lds, &grid))) return rc;
    if (nq > (u64)grid) {
        // several rounds of waves: as many waves as make the rounds equally full (10,000 queries on 4,096 waves: 3,334),
        // instead of a last round that leaves most of the GPU idle
        const u64 rounds = (nq + (u64)grid - 1) / (u64)grid;
        grid = (int)((nq + rounds - 1) / rounds);
    }
    a.qrot = ix->ws_qrot; a.tables = ix->ws_tab;
    a.nq = (u32)nq; a.K = K;
    a.out_ids = (long long*)ids; a.out_dists = dists;
    a.out_scale = ix->metric == PAG_L2 ? 1.0f : 0.5f;
    // A record caught between two states of a reverse-edge pass (its id row can span two cache lines, and a node may
    // change slots) can show one node twice; the merge needs the keys of a hop distinct.
    if (ix->concurrent_view) a.flags |= PAG_SEARCH_DISTINCT;
    PAG_HIP(hipEventRecord(ix->ev[0], ix->stream));
    if ((rc = prepare(ix, Q, nq, ix->ws_qrot, ix->ws_tab))) return rc;
    // more queries than resident waves: those that run side by side are chosen to be neighbours
    if (!(ix->flags & PAG_FLAG_KEEP_QUERY_ORDER) && nq > (u64)grid && (rc = pag_order_queries(ix, ix->ws_qrot, nq, &a.order))) return rc;
    if ((rc = pag_launch_zero_u32(ix->stream, ix->d_qcounter, 1))) return rc;
    PAG_HIP(hipEventRecord(ix->ev[1], ix->stream));
    if ((rc = pag_launch_search(ix, a, lds, &grid))) return rc;
    PAG_HIP(hipEventRecord(ix->ev[2], ix->stream));
    PAG_HIP(hipStreamSynchronize(ix->stream));
    float ms = 0.f;
    PAG_HIP(hipEventElapsedTime(&ms, ix->ev[0], ix->ev[1])); ix->last_prepare_ms = ms;
    PAG_HIP(hipEventElapsedTime(&ms, ix->ev[1], ix->ev[2])); ix->last_search_ms = ms;
    return PAG_OK;
}

extern "C" int pag_search(const pag_index* cix, const float* Q, uint64_t nq, uint32_t K, uint32_t efS,
                          int64_t* ids, float* dists) {
    pag_index* ix = const_cast<pag_index*>(cix);   // workspaces and counters are mutable state of the handle
    PAG_CHECK(ix != nullptr, PAG_EINVAL, "index is null");
    return search_impl(ix, Q, nq, K, efS, ids, dists);
}

// ---------------------------------------------------------------------------------------------
// pag_search_static: pag_search for callers that cannot allocate.  Everything the search needs beyond the index, the
// queries and the outputs -- rotated queries, projection tables, normalised copies (COS) and the per-wave seen-set
// bitmaps -- lives in one file-scope device array.  Each GPU holds its own copy of that array, at its own address,
// until the process ends; the address is looked up once per device.
extern "C" int pag_search_static(const pag_index* cix, const float* Q, uint64_t nq, uint32_t K, uint32_t efS,
                                 int64_t* ids, float* dists) {
    pag_index* ix = const_cast<pag_index*>(cix);
    PAG_CHECK(ix != nullptr, PAG_EINVAL, "index is null");
    if (nq == 0) return PAG_OK;
    PAG_CHECK(Q && ids && dists, PAG_EINVAL, "Q, ids or dists is null");
    PAG_CHECK(K >= 1 && K <= ix->n, PAG_EINVAL, "K must be in 1..n");
    PAG_CHECK(efS >= 1, PAG_EINVAL, "efS must be >= 1");
    const u32 b = ix->search_b ? ix->search_b : std::max<u32>(10, K);
    PAG_CHECK(b >= K, PAG_EINVAL, "search_b must be >= K");
    PAG_CHECK(b <= PAG_LDS_RING_MAX_B, PAG_EUNSUPPORTED,
              "pag_search_static: working sets above 128 nodes (K > 128) keep their rings in a workspace; use pag_search");
    DeviceGuard g(ix->device);
    const pag_layout& L = ix->L;
    // query part: rotated queries, tables, normalised copies; each block starts on a 256-byte boundary
    const u64 per_query = (u64)L.d + (u64)L.Ppad * PAG_NCODE + (ix->metric == PAG_COS ? L.d : 0);
    PAG_CHECK(nq <= PAG_STATIC_QUERY_FLOATS / per_query, PAG_EUNSUPPORTED,
              "pag_search_static: nq * (d + 16 * subspaces [+ d for cosine]) exceeds 4,194,304 floats; split the batch or use pag_search");
    auto align256 = [](u64 x) { return (x + 255) / 256 * 256; };
    const u64 off_qrot = 0;
    const u64 off_tab = align256(off_qrot + nq * L.d * 4);
    const u64 off_norm = align256(off_tab + nq * L.Ppad * PAG_NCODE * 4);
    const u64 off_bitmap = align256(off_norm + (ix->metric == PAG_COS ? nq * L.d * 4 : 0));
    int rc;
    SearchArgs a;
    u32 lds = 0;
    int grid = 0;
    if ((rc = search_plan(ix, b, efS, ix->n, &a, &lds, &grid))) return rc;
    // bitmap part: as many per-wave bitmaps as fit behind the query part; fewer waves than the GPU could hold
    // make the search slower, not different
    const u64 room = (u64)PAG_STATIC_SCRATCH_BYTES - off_bitmap;
    const u64 fit = room / (a.bitmap_words * 4);
    PAG_CHECK(fit >= 64, PAG_EUNSUPPORTED,
              "pag_search_static: the index capacity is too large for the static seen-set bitmaps (4,194,304 vectors at most); use pag_search");
    if ((u64)grid > fit) grid = (int)fit;
    if ((u64)grid > nq) grid = (int)nq;
    unsigned char* base = nullptr;
    if ((rc = scratch_of(ix->device, &base))) return rc;
    a.qrot = (const float*)(base + off_qrot);
    a.tables = (const float*)(base + off_tab);
    a.bitmap = (u32*)(base + off_bitmap);
    a.nq = (u32)nq; a.K = K;
    a.out_ids = (long long*)ids; a.out_dists = dists;
    a.out_scale = ix->metric == PAG_L2 ? 1.0f : 0.5f;
    PAG_HIP(hipEventRecord(ix->ev[0], ix->stream));
    // the array keeps whatever the last call left there, possibly under another layout: the bitmaps start clean
    if ((rc = pag_launch_zero_u32(ix->stream, a.bitmap, (u64)grid * a.bitmap_words))) return rc;
    if ((rc = prepare_into(ix, Q, nq, (float*)(base + off_norm), (float*)(base + off_qrot), (float*)(base + off_tab)))) return rc;
    if ((rc = pag_launch_zero_u32(ix->stream, ix->d_qcounter, 1))) return rc;
    PAG_HIP(hipEventRecord(ix->ev[1], ix->stream));
    if ((rc = pag_launch_search(ix, a, lds, &grid))) return rc;
    PAG_HIP(hipEventRecord(ix->ev[2], ix->stream));
    PAG_HIP(hipStreamSynchronize(ix->stream));
    float ms = 0.f;
    PAG_HIP(hipEventElapsedTime(&ms, ix->ev[0], ix->ev[1])); ix->last_prepare_ms = ms;
    PAG_HIP(hipEventElapsedTime(&ms, ix->ev[1], ix->ev[2])); ix->last_search_ms = ms;
    return PAG_OK;
}

// ---------------------------------------------------------------------------------------------
// Searchers: a view of an index with workspaces, counters, events and a stream of its own, so that
// searches can run while pag_insert (or another searcher) works on the same index.
struct pag_searcher {
    pag_index view;             // shares the parent's HBM-resident index, owns everything else
    const pag_index* parent;
};

static void searcher_release(pag_searcher* s) {
    pag_index& v = s->view;
    void* ptrs[] = { v.ws_qrot, v.ws_tab, v.ws_norm, v.ws_bitmap, v.ws_rings, v.ws_order, v.d_qcounter, v.d_counters };
    for (void* p : ptrs) if (p) (void)hipFree(p);
    for (auto& e : v.ev) if (e) (void)hipEventDestroy(e);
    delete s;
}

extern "C" int pag_searcher_create(const pag_index* ix, void* stream, pag_searcher** out) {
    PAG_CHECK(out != nullptr, PAG_EINVAL, "out is null");
    *out = nullptr;
    PAG_CHECK(ix != nullptr, PAG_EINVAL, "index is null");
    DeviceGuard g(ix->device);
    pag_searcher* s = new pag_searcher();
    s->parent = ix;
    s->view = *ix;
    pag_index& v = s->view;
    v.stream = (hipStream_t)stream;
    v.concurrent_view = 1;
    v.ws_qrot = nullptr; v.ws_qrot_cap = 0;
    v.ws_tab = nullptr; v.ws_tab_cap = 0;
    v.ws_norm = nullptr; v.ws_norm_cap = 0;
    v.ws_bitmap = nullptr; v.ws_bitmap_cap = 0;
    v.ws_rings = nullptr; v.ws_rings_cap = 0;
    v.ws_order = nullptr; v.ws_order_cap = 0;
    v.d_qcounter = nullptr; v.d_counters = nullptr;
    for (auto& e : v.ev) e = nullptr;
    v.last_search_ms = v.last_prepare_ms = v.last_build_ms = 0.0;
    int rc;
    if ((rc = dev_alloc(&v.d_qcounter, 4)) || (rc = dev_alloc(&v.d_counters, CTR_COUNT))) { searcher_release(s); return rc; }
    hipError_t e = hipMemsetAsync(v.d_counters, 0, CTR_COUNT * sizeof(u64), v.stream);
    for (auto& ev : v.ev) if (e == hipSuccess) e = hipEventCreate(&ev);
    if (e == hipSuccess) e = hipStreamSynchronize(v.stream);
    if (e != hipSuccess) { searcher_release(s); pag_set_error(std::string("pag_searcher_create: ") + hipGetErrorString(e)); return PAG_EHIP; }
    *out = s;
    return PAG_OK;
}

extern "C" int pag_searcher_search(pag_searcher* s, const float* Q, uint64_t nq, uint32_t K, uint32_t efS,
                                   int64_t* ids, float* dists) {
    PAG_CHECK(s != nullptr, PAG_EINVAL, "searcher is null");
    const pag_index* p = s->parent;
    // the nodes whose insertion has completed: pag_insert publishes n after its last kernel has finished
    s->view.n = __atomic_load_n(&p->n, __ATOMIC_ACQUIRE);
    s->view.n_entry = p->n_entry;
    s->view.search_b = p->search_b;
    s->view.flags = p->flags;
    s->view.seen_log2 = p->seen_log2;
    return search_impl(&s->view, Q, nq, K, efS, ids, dists);
}

extern "C" int pag_searcher_get_counters(const pag_searcher* s, pag_counters* out) {
    PAG_CHECK(s != nullptr, PAG_EINVAL, "searcher is null");
    return pag_get_counters(&s->view, out);
}

extern "C" int pag_searcher_free(pag_searcher* s) {
    if (!s) return PAG_OK;
    DeviceGuard g(s->view.device);
    (void)hipStreamSynchronize(s->view.stream);
    searcher_release(s);
    return PAG_OK;
}

extern "C" int pag_prepare_queries(const pag_index* cix, const float* Q, uint64_t nq, float* q_rot, float* tables) {
    pag_index* ix = const_cast<pag_index*>(cix);
    PAG_CHECK(ix && Q && q_rot && tables, PAG_EINVAL, "null argument");
    DeviceGuard g(ix->device);
    const pag_layout& L = ix->L;
    int rc;
    // the search keeps zero-padded tables of Ppad rows; this entry point returns the P real rows
    if ((rc = ensure_ws(&ix->ws_tab, &ix->ws_tab_cap, nq * L.Ppad * PAG_NCODE))) return rc;
    if ((rc = prepare(ix, Q, nq, q_rot, ix->ws_tab))) return rc;
    PAG_HIP(hipMemcpy2DAsync(tables, (size_t)L.P * PAG_NCODE * 4, ix->ws_tab, (size_t)L.Ppad * PAG_NCODE * 4,
                             (size_t)L.P * PAG_NCODE * 4, nq, hipMemcpyDeviceToDevice, ix->stream));
    PAG_HIP(hipStreamSynchronize(ix->stream));
    return PAG_OK;
}

extern "C" int pag_exact_distances(const pag_index* ix, const float* q_rot, uint64_t nq, const uint32_t* ids,
                                   uint32_t m, float* keys) {
    PAG_CHECK(ix && q_rot && ids && keys, PAG_EINVAL, "null argument");
    DeviceGuard g(ix->device);
    int rc = pag_launch_exact(ix->stream, ix, q_rot, nq, ids, m, keys);
    if (rc) return rc;
    PAG_HIP(hipStreamSynchronize(ix->stream));
    return PAG_OK;
}

extern "C" int pag_screen(const pag_index* cix, const float* tables, uint64_t nq, const uint32_t* u,
                          const float* Du, float* est) {
    pag_index* ix = const_cast<pag_index*>(cix);
    PAG_CHECK(ix && tables && u && Du && est, PAG_EINVAL, "null argument");
    DeviceGuard g(ix->device);
    const pag_layout& L = ix->L;
    int rc;
    // widen the caller's [P][16] tables to the zero-padded [Ppad][16] form the kernels read
    if ((rc = ensure_ws(&ix->ws_tab, &ix->ws_tab_cap, nq * L.Ppad * PAG_NCODE))) return rc;
    PAG_HIP(hipMemsetAsync(ix->ws_tab, 0, nq * L.Ppad * PAG_NCODE * 4, ix->stream));
    PAG_HIP(hipMemcpy2DAsync(ix->ws_tab, (size_t)L.Ppad * PAG_NCODE * 4, tables, (size_t)L.P * PAG_NCODE * 4,
                             (size_t)L.P * PAG_NCODE * 4, nq, hipMemcpyDeviceToDevice, ix->stream));
    if ((rc = pag_launch_screen(ix->stream, ix, ix->ws_tab, nq, u, Du, est))) return rc;
    PAG_HIP(hipStreamSynchronize(ix->stream));
    return PAG_OK;
}

static int edge_info_impl(const pag_index* cix, uint64_t node_begin, uint64_t node_end, uint8_t* codes,
                          float* a, float* c, float* e2) {
    pag_index* ix = const_cast<pag_index*>(cix);
    PAG_CHECK(ix && codes && a && c && e2, PAG_EINVAL, "null argument");
    PAG_CHECK(node_begin <= node_end && node_end <= ix->n, PAG_EINVAL, "node range out of bounds");
    if (node_begin == node_end) return PAG_OK;
    DeviceGuard g(ix->device);
    const pag_layout& L = ix->L;
    const u64 m = node_end - node_begin;
    // work on a scratch copy of the records so that the index itself is left untouched
    uint8_t* srec = nullptr;
    float* se2 = nullptr;
    int rc;
    std::vector<uint8_t> buf(m * L.rec_bytes);      // host staging before anything is held on the device
    std::vector<float> he2(m * L.deg);
    if ((rc = dev_alloc(&srec, m * L.rec_bytes))) return rc;
    if ((rc = dev_alloc(&se2, m * L.deg))) { (void)hipFree(srec); return rc; }
    hipError_t e = hipMemcpyAsync(srec, ix->rec + node_begin * L.rec_bytes, m * L.rec_bytes, hipMemcpyDeviceToDevice, ix->stream);
    if (e == hipSuccess) rc = pag_launch_edge_info_nodes(ix->stream, ix, node_begin, node_end, srec, se2, node_begin);
    if (e == hipSuccess && rc == PAG_OK) e = hipStreamSynchronize(ix->stream);
    if (e == hipSuccess && rc == PAG_OK) e = hipMemcpy(buf.data(), srec, buf.size(), hipMemcpyDeviceToHost);
    if (e == hipSuccess && rc == PAG_OK) e = hipMemcpy(he2.data(), se2, he2.size() * 4, hipMemcpyDeviceToHost);
    (void)hipFree(srec); (void)hipFree(se2);
    if (rc) return rc;
    if (e != hipSuccess) { pag_set_error(std::string("pag_edge_info: ") + hipGetErrorString(e)); return PAG_EHIP; }
    for (u64 i = 0; i < m; ++i) {
        const uint8_t* rec = buf.data() + i * L.rec_bytes;
        std::memcpy(a + i * L.deg, rec + L.off_a, L.deg * 4);
        std::memcpy(c + i * L.deg, rec + L.off_c, L.deg * 4);
        std::memcpy(e2 + i * L.deg, he2.data() + i * L.deg, L.deg * 4);
        const u32* cw = (const u32*)(rec + L.off_codes);
        for (u32 ed = 0; ed < L.deg; ++ed)
            for (u32 l = 0; l < L.P; ++l)
                codes[(i * L.deg + ed) * L.P + l] = (uint8_t)((cw[ed * L.cw + l / 8] >> (4 * (l % 8))) & 15u);
    }
    return PAG_OK;
}

extern "C" int pag_edge_info(const pag_index* cix, uint64_t node_begin, uint64_t node_end, uint8_t* codes,
                             float* a, float* c, float* e2) {
    return guarded("pag_edge_info", [&]() { return edge_info_impl(cix, node_begin, node_end, codes, a, c, e2); });
}

extern "C" int pag_measure_row_reads(const pag_index* cix, uint64_t rows, int scattered, double* gb_per_s) {
    pag_index* ix = const_cast<pag_index*>(cix);
    PAG_CHECK(ix && gb_per_s, PAG_EINVAL, "null argument");
    PAG_CHECK(rows >= 1 && ix->n >= 1, PAG_EINVAL, "rows must be >= 1");
    PAG_CHECK(scattered >= 0 && scattered <= 2, PAG_EINVAL, "mode must be 0, 1 or 2");
    PAG_CHECK(((u64)ix->L.d * (ix->vec_half ? 2 : 4)) % 16 == 0, PAG_EUNSUPPORTED, "rows must be a multiple of 16 bytes");
    DeviceGuard g(ix->device);
    // a multiplier coprime with n makes (counter * stride) mod n a permutation of the rows
    u64 stride = 0;
    if (scattered) {
        stride = (u64)(0.6180339887 * (double)ix->n) | 1ull;
        auto gcd = [](u64 a, u64 b) { while (b) { u64 t = a % b; a = b; b = t; } return a; };
        while (gcd(stride, ix->n) != 1) stride += 2;
    }
    const int grid = ix->num_cu * 16;
    int rc;
    if (scattered == 2) {
        // the traffic of whole hops: rows / 7 hops of 7 rows, one record, 8 bitmap reads, 7 bitmap writes each
        const u64 words = ((u64)ix->capacity + 127) / 128 * 4;
        const u64 need = (u64)grid * words;
        if (ix->ws_bitmap_cap < need) {
            if ((rc = ensure_ws(&ix->ws_bitmap, &ix->ws_bitmap_cap, need))) return rc;
            PAG_HIP(hipMemsetAsync(ix->ws_bitmap, 0, need * 4, ix->stream));
        }
        const u64 hops = std::max<u64>(1, rows / 7);
        for (int rep = 0; rep < 2; ++rep) {
            PAG_HIP(hipEventRecord(ix->ev[0], ix->stream));
            if ((rc = pag_launch_hop_traffic(ix->stream, ix, hops, ix->ws_bitmap, words, ix->d_qcounter + 1, grid))) return rc;
            PAG_HIP(hipEventRecord(ix->ev[1], ix->stream));
            PAG_HIP(hipStreamSynchronize(ix->stream));
        }
        // searches expect clean bitmaps
        PAG_HIP(hipMemsetAsync(ix->ws_bitmap, 0, need * 4, ix->stream));
        PAG_HIP(hipStreamSynchronize(ix->stream));
        float ms2 = 0.f;
        PAG_HIP(hipEventElapsedTime(&ms2, ix->ev[0], ix->ev[1]));
        *gb_per_s = (double)hops * (7.0 * ix->L.d * (ix->vec_half ? 2 : 4) + ix->L.rec_bytes) / ((double)ms2 * 1e6);
        return PAG_OK;
    }
    for (int rep = 0; rep < 2; ++rep) {      // first pass warms up, second is timed
        PAG_HIP(hipEventRecord(ix->ev[0], ix->stream));
        if ((rc = pag_launch_row_reads(ix->stream, ix, rows, stride, ix->d_qcounter + 1, grid))) return rc;
        PAG_HIP(hipEventRecord(ix->ev[1], ix->stream));
        PAG_HIP(hipStreamSynchronize(ix->stream));
    }
    float ms = 0.f;
    PAG_HIP(hipEventElapsedTime(&ms, ix->ev[0], ix->ev[1]));
    *gb_per_s = (double)rows * ix->L.d * (ix->vec_half ? 2 : 4) / ((double)ms * 1e6);
    return PAG_OK;
}
