// Instantiations of the search kernel: stored vectors of up to 3 chunks per lane (fp32 rows of
// up to 768 elements; 16-bit rows of up to 1536 elements in 16-byte chunks or 768 in 8-byte chunks),
// 8 code dwords per neighbour (up to 64 subspaces).
#include "pag_search_kernel.h"

PAG_SEARCH_INSTANCES(3, 8)
