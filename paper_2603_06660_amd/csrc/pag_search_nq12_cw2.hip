// Instantiations of the search kernel: stored vectors of up to 12 16-byte chunks per lane
// (fp32 rows of up to 3072 elements, 16-bit rows of up to 6144), 2 code dwords per neighbour.
#include "pag_search_kernel.h"

PAG_SEARCH_INSTANCES(12, 2)
