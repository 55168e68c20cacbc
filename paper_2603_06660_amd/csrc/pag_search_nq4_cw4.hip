// Instantiations of the search kernel: stored vectors of up to 4 16-byte chunks per lane
// (fp32 rows of up to 1024 elements, 16-bit rows of up to 2048), 4 code dwords per neighbour.
#include "pag_search_kernel.h"

PAG_SEARCH_INSTANCES(4, 4)
