// Instantiations of the search kernel: stored vectors of up to 8 16-byte chunks per lane
// (fp32 rows of up to 2048 elements, 16-bit rows of up to 4096), 2 code dwords per neighbour.
#include "pag_search_kernel.h"

typedef void (*pag_search_fn)(const SearchArgs);
pag_search_fn pag_search_fn_nq8_cw2(int nw, bool half) {
    if (half) return nullptr;
    return nw == 1 ? (pag_search_fn)pagk::k_search<8, 1, false, 2> : (pag_search_fn)pagk::k_search<8, 2, false, 2>;
}
