// Instantiations of the search kernel: stored vectors of up to 8 16-byte chunks per lane
// (fp32 rows of up to 2048 elements, 16-bit rows of up to 4096), 2 code dwords per neighbour.
#include "pag_search_kernel.h"

PAG_SEARCH_INSTANCES(8, 2)
