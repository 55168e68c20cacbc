// Instantiations of the search kernel: stored vectors of up to 6 chunks per lane (fp32 rows of
// up to 1536 elements; 16-bit rows of up to 3072 elements in 16-byte chunks or 1536 in 8-byte chunks),
// 4 code dwords per neighbour (up to 32 subspaces).
#include "pag_search_kernel.h"

PAG_SEARCH_INSTANCES(6, 4)
