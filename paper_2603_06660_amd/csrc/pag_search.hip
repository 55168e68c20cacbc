// Launch logic of the search kernel: picks the instantiation for (d, b), sizes the per-wave LDS
// carve-up and the persistent grid.
#include "pag_internal.h"

typedef void (*pag_search_fn)(const SearchArgs);   // selectors: one per (row chunks per lane, code dwords)
pag_search_fn pag_search_fn_nq1_cw2(int, int);
pag_search_fn pag_search_fn_nq1_cw4(int, int);
pag_search_fn pag_search_fn_nq1_cw8(int, int);
pag_search_fn pag_search_fn_nq2_cw2(int, int);
pag_search_fn pag_search_fn_nq2_cw4(int, int);
pag_search_fn pag_search_fn_nq2_cw8(int, int);
pag_search_fn pag_search_fn_nq3_cw2(int, int);
pag_search_fn pag_search_fn_nq3_cw4(int, int);
pag_search_fn pag_search_fn_nq3_cw8(int, int);
pag_search_fn pag_search_fn_nq4_cw2(int, int);
pag_search_fn pag_search_fn_nq4_cw4(int, int);
pag_search_fn pag_search_fn_nq4_cw8(int, int);
pag_search_fn pag_search_fn_nq6_cw2(int, int);
pag_search_fn pag_search_fn_nq6_cw4(int, int);
pag_search_fn pag_search_fn_nq6_cw8(int, int);
pag_search_fn pag_search_fn_nq8_cw2(int, int);
pag_search_fn pag_search_fn_nq8_cw4(int, int);
pag_search_fn pag_search_fn_nq8_cw8(int, int);
pag_search_fn pag_search_fn_nq10_cw2(int, int);
pag_search_fn pag_search_fn_nq10_cw4(int, int);
pag_search_fn pag_search_fn_nq10_cw8(int, int);
pag_search_fn pag_search_fn_nq12_cw2(int, int);
pag_search_fn pag_search_fn_nq12_cw4(int, int);
pag_search_fn pag_search_fn_nq12_cw8(int, int);

static pag_search_fn pick(u32 d, u32 b, bool half, u32 cw) {
    int nw = 1;                                       // entries of W per lane: 64 * nw >= b
    while (64u * nw < b) nw *= 2;
    // how a row is cut into per-lane chunks: fp32 rows in 16-byte chunks (256 elements per chunk
    // row); 16-bit rows in 16-byte chunks (512 elements) or, when that would leave more of the last
    // chunk row empty, in 8-byte chunks (256 elements)
    int vm = 0;
    u32 per_chunk_row = 256;
    if (half) {
        const u32 waste16 = (d + 511) / 512 * 512 - d, waste8 = (d + 255) / 256 * 256 - d;
        vm = waste8 < waste16 ? 2 : 1;
        per_chunk_row = vm == 1 ? 512 : 256;
    }
    // chunk rows a stored row needs; the kernel for `chunks` rows or, where that count is not instantiated,
    // for one more (it masks its last two chunk rows): 1, 2, 3, 4, 6, 8, 10, 12
    const u32 chunks = (d + per_chunk_row - 1) / per_chunk_row;
#define PAG_PICK_CW(NQ)                                              \
    switch (cw) {                                                    \
        case 2: return pag_search_fn_nq##NQ##_cw2(nw, vm);         \
        case 4: return pag_search_fn_nq##NQ##_cw4(nw, vm);         \
        case 8: return pag_search_fn_nq##NQ##_cw8(nw, vm);         \
        default: return nullptr;                                     \
    }
    if (chunks <= 1) { PAG_PICK_CW(1) }
    if (chunks <= 2) { PAG_PICK_CW(2) }
    if (chunks <= 3) { PAG_PICK_CW(3) }
    if (chunks <= 4) { PAG_PICK_CW(4) }
    if (chunks <= 6) { PAG_PICK_CW(6) }
    if (chunks <= 8) { PAG_PICK_CW(8) }
    if (chunks <= 10) { PAG_PICK_CW(10) }
    if (chunks <= 12) { PAG_PICK_CW(12) }
#undef PAG_PICK_CW
    return nullptr;
}

static u32 align_up(u32 x, u32 a) { return (x + a - 1) / a * a; }

// LDS carve-up of one wave; fills the offsets in `a` and returns the total.
int pag_search_lds_bytes(const pag_layout& L, u32 b, u32 hlog, u32 blog, SearchArgs* a) {
    u32 off = align_up(L.Ppad * PAG_NCODE * 4, 16);
    a->off_hash = off; off += (4u << hlog);
    a->off_bloom = off; off += blog ? (1u << blog) / 8 : 0;
    // round ends sort up to 2b keys: working sets of up to 128 nodes by ranks from SA into SB, both in LDS;
    // larger ones in registers (no LDS)
    u32 sa = 2 * b, sb = 2 * b;
    if (b > PAG_LDS_RING_MAX_B) sa = sb = 0;
    a->off_sa = off;   off += align_up(sa * 8, 16);
    a->off_sb = off;   off += align_up(sb * 8, 16);
    u32 ring = 32;                                    // the last b pushes must stay apart: any power of two >= b
    while (ring < b) ring *= 2;
    a->ring_mask = ring - 1;
    const u32 ring_lds = b > PAG_LDS_RING_MAX_B ? 0 : ring * 8;   // above that the rings live in HBM
    a->off_rf = off;   off += ring_lds;
    a->off_rt = off;   off += ring_lds;
    return (int)off;
}

int pag_search_max_grid(const pag_index* ix, u32 b, u32 lds_bytes, int* grid) {
    pag_search_fn fn = pick(ix->L.d, b, ix->vec_half != 0, ix->L.cw);
    if (!fn) { pag_set_error("search: dimension above 3072 is not built"); return PAG_EUNSUPPORTED; }
    int per_cu = 0;
    PAG_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void*)fn, 64, lds_bytes));
    if (per_cu < 1) per_cu = 1;
    *grid = per_cu * ix->num_cu;
    return PAG_OK;
}

int pag_launch_search(const pag_index* ix, const SearchArgs& a, u32 lds_bytes, int* grid_io) {
    pag_search_fn fn = pick(a.d, a.b, ix->vec_half != 0, a.cw);
    if (!fn) { pag_set_error("search: dimension above 3072 is not built"); return PAG_EUNSUPPORTED; }
    int grid = *grid_io;
    if ((u64)grid > a.nq) grid = (int)a.nq;
    if (grid < 1) return PAG_OK;
    SearchArgs args = a;
    void* kargs[] = { (void*)&args };
    PAG_HIP(hipLaunchKernel((const void*)fn, dim3(grid), dim3(64), kargs, lds_bytes, ix->stream));
    *grid_io = grid;
    return PAG_OK;
}
