// Instantiations of the search kernel: stored vectors of up to 3 16-byte chunks per lane
// (fp32 rows of up to 768 elements, 16-bit rows of up to 1536), 2 code dwords per neighbour.
#include "pag_search_kernel.h"

typedef void (*pag_search_fn)(const SearchArgs);
pag_search_fn pag_search_fn_nq3_cw2(int nw, bool half) {
    if (half) return nw == 1 ? (pag_search_fn)pagk::k_search<3, 1, true, 2> : (pag_search_fn)pagk::k_search<3, 2, true, 2>;
    return nw == 1 ? (pag_search_fn)pagk::k_search<3, 1, false, 2> : (pag_search_fn)pagk::k_search<3, 2, false, 2>;
}
