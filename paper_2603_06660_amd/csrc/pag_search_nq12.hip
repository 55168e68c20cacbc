// Instantiation of the search kernel for vectors of up to 3072 floats (12 float4 per lane).
#include "pag_search_kernel.h"

typedef void (*pag_search_fn)(const SearchArgs);
pag_search_fn pag_search_fn_nq12(int nw) {
    return nw == 1 ? (pag_search_fn)pagk::k_search<12, 1> : (pag_search_fn)pagk::k_search<12, 2>;
}
