"""MI355X-native PAG (Projection-Augmented Graph) search: thin Python binding over the C ABI.

    from paper_2603_06660_amd import PagIndex
    ix = PagIndex.build(base_cuda, metric="ip", max_degree=32, num_subspaces=32, ef_construction=100)
    ids, dists = ix.search(queries_cuda, K=10, efS=64)

All computation runs in libpag_hip.so (hand-written HIP kernels for gfx950); torch only
provides device memory and the stream.  Importing this package does not load the library;
the first use does, and raises if it has not been built.
"""
from .binding import (PagIndex, PagError, load_library, library_path, EXPORTED_SYMBOLS,  # noqa: F401
                      L2, IP, COS, FLAG_NO_PRT, FLAG_NO_PES, FLAG_FP16_VECTORS, FLAG_KEEP_ORDER,
                      FLAG_EXACT_TEST_COUNT, FLAG_PERMUTATION_TRANSFORM, FLAG_KEEP_QUERY_ORDER)
