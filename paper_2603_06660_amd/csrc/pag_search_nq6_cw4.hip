// Instantiations of the search kernel: stored vectors of up to 6 16-byte chunks per lane
// (fp32 rows of up to 1536 elements, 16-bit rows of up to 3072), 4 code dwords per neighbour.
#include "pag_search_kernel.h"

PAG_SEARCH_INSTANCES(6, 4)
