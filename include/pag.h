/*
 * pag.h -- C ABI of the MI355X (gfx950) PAG library.
 *
 * PAG (Projection-Augmented Graph) answers approximate K-nearest-neighbour
 * queries over a dataset D of n vectors in R^d (problem statement, Sec. 1) with
 * a best-first search over a proximity graph in which a projection-based test
 * (PRT, Eq. 3, with the Test-Feedback-Buffer threshold of Eq. 4) decides which
 * neighbours get an exact distance (Alg. 2).  The index is built by inserting
 * the vectors with that same search followed by RobustPrune (Alg. 1, Step 1;
 * Eq. 1).
 *
 * Conventions for every entry point
 *   - "dev" pointers are device (HBM) pointers of the GPU that was current when
 *     the index was created; "host" pointers are ordinary host memory.  All
 *     buffers are row-major, contiguous and owned by the caller: the library
 *     never frees them and copies whatever it keeps, so they may be released
 *     as soon as the call returns.
 *   - Work is enqueued on pag_params.stream (a hipStream_t, NULL = the null
 *     stream) and every call returns after that stream has been synchronised.
 *   - Return value: PAG_OK (0) or a negative pag_status; pag_last_error()
 *     returns a thread-local, human readable description of the last failure.
 *     No exception crosses this boundary.
 *   - Node ids are the row numbers of the vectors in insertion order.
 *   - A handle owns workspaces and counters: calls on one index must not overlap in time
 *     (different indexes are independent).  The exception is a pag_searcher, which has
 *     workspaces, counters and a stream of its own: pag_searcher_search may run while
 *     pag_insert, pag_search or other searchers work on the same index.
 */
#ifndef PAG_H
#define PAG_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pag_index pag_index; /* opaque; created by pag_build / pag_import, destroyed by pag_free */

typedef enum { PAG_L2 = 0, PAG_IP = 1, PAG_COS = 2 } pag_metric;

typedef enum {
    PAG_OK = 0,
    PAG_EINVAL = -1,       /* null / inconsistent argument, d % num_subspaces != 0, K == 0, K > n ... */
    PAG_ECAPACITY = -2,    /* pag_insert beyond pag_params.capacity */
    PAG_ENOMEM = -3,       /* host or device allocation failed */
    PAG_EHIP = -4,         /* a HIP call failed; text in pag_last_error() */
    PAG_EUNSUPPORTED = -5  /* a size outside what the kernels are built for (see pag_params) */
} pag_status;

/*
 * Index parameters (Alg. 1 inputs; Appendix D).  Names in brackets are the
 * paper's.  Limits of this build: d % 4 == 0, d <= 3072, num_subspaces <= 64,
 * d % num_subspaces == 0, max_degree <= 64, working-set size b <= 1024.
 */
typedef struct {
    uint32_t struct_size;     /* sizeof(pag_params), for ABI checking */
    int32_t  metric;          /* pag_metric.  PAG_IP expects unit-norm vectors (it ranks like PAG_COS
                                 without normalising); PAG_COS normalises base vectors and queries. */
    uint32_t max_degree;      /* [2M] maximum out-degree */
    uint32_t num_subspaces;   /* [L] number of subspaces of the rotated space; 16 projection vectors each */
    uint32_t ef_construction; /* [efC] nodes visited per insertion; W has min(efC, 100) nodes while indexing */
    uint32_t search_b;        /* working-set size b = |W| when searching; 0 = max(10, K) (Alg. 2) */
    uint32_t insert_subbatch; /* vectors inserted concurrently per step of the batch-synchronous build; 0 = auto;
                                 at most 2^20 */
    uint32_t flags;           /* PAG_FLAG_* */
    uint64_t capacity;        /* maximum number of vectors including later pag_insert calls; 0 = n */
    uint64_t seed;            /* seed of the random transform Q and of the codebooks */
    void*    stream;          /* hipStream_t; NULL = null stream */
} pag_params;

#define PAG_FLAG_NO_PRT 1u    /* ablation: skip the projection test, every unseen neighbour gets an exact distance */
#define PAG_FLAG_FP16_VECTORS 4u /* keep the rotated base vectors as 16-bit floats (the paper's payload, Sec. 4.2): halves the
                                   bytes per exact distance; the index then *is* the rounded data, and all arithmetic on it
                                   stays fp32/fp64.  Needs d % 8 == 0.  Build / import time only. */
#define PAG_FLAG_NO_PES 2u    /* ablation: index without the PES candidate buffers H(v) (Eq. 5; Alg. 1's last loop) */
#define PAG_FLAG_KEEP_ORDER 8u /* build / insert link the vectors in the order given (row 0 first) instead of a
                                  seeded shuffle: for input that is already in random order.  With
                                  insert_subbatch = 1 this is Alg. 1 as printed, one node after another, the
                                  PES buffer of a node verified right after its insertion. */
#define PAG_FLAG_EXACT_TEST_COUNT 16u /* diagnostic, search time: long searches resolve the seen set for every
                                  neighbour before the projection test instead of only for those that pass it,
                                  so that pag_counters.tests counts exactly the unseen neighbours (Sec. 4.2's
                                  gamma = passes / tests).  Results are unchanged; the search is a few % slower. */
#define PAG_FLAG_PERMUTATION_TRANSFORM 32u /* build time: Q is a random signed permutation (a coordinate shuffle with random
                                  signs) instead of a Haar-distributed rotation.  Still orthogonal, and its products are exact,
                                  so the stored vectors are the input's values bit for bit; it does not mix coordinates, so
                                  it suits data that is already isotropic (and comparisons that must not depend on rounding). */
#define PAG_FLAG_KEEP_QUERY_ORDER 64u /* search time: the queries of a call are taken as numbered.  By default a call with more
                                  queries than the GPU keeps waves resident takes them in the order of their projections onto
                                  the batch's direction of largest spread, so that searches running side by side visit the
                                  same part of the graph and share rows in the caches.  Results never depend on it. */

/*
 * Flat host view of an index (Alg. 1 output: node set, edge set E, inference
 * structure I, transform Q, codebooks).  Used by pag_export (the library fills
 * caller-allocated arrays) and pag_import (the library copies from them).
 */
typedef struct {
    uint32_t struct_size;
    int32_t  metric;
    uint64_t n;
    uint32_t d;
    uint32_t num_subspaces;   /* P */
    uint32_t max_degree;      /* deg */
    uint32_t n_entry;
    float*    vectors;   /* host [n*d]        base vectors after normalisation (COS) and rotation by Q (and rounding
                                              to 16-bit floats with PAG_FLAG_FP16_VECTORS), as fp32 */
    uint32_t* adj;       /* host [n*deg]      out-neighbour ids; 0xFFFFFFFF = free slot */
    float*    a;         /* host [n*deg]      a_i = ||w_i-u|| / cos(beta_i)            (Sec. 3.1) */
    float*    c;         /* host [n*deg]      c_i = ||w_i-u||^2 + 2 a_i sum_l <u_l, r*_il>  (stored offsets, Appendix C) */
    float*    e2;        /* host [n*deg]      ||w_i-u||^2 */
    uint8_t*  codes;     /* host [n*deg*P]    index (0..15) of the selected reference vector per subspace */
    float*    rotation;  /* host [d*d]        Q, row-major; rotated = Q x */
    float*    codebooks; /* host [P*16*(d/P)] projection vectors r_jl, norm 1/sqrt(P) */
    uint32_t* entry;     /* host [n_entry]    entry node ids; a search starts from the first b of them */
} pag_arrays;

/* Sums over all searches since creation or the last pag_reset_counters (Sec. 4.2's quantities); the searches
 * that pag_build and pag_insert run for their own vectors count as well. */
typedef struct {
    uint32_t struct_size;
    uint32_t adj_record_bytes;   /* size of one node's adjacency record in HBM */
    uint64_t queries;
    uint64_t hops;               /* expanded nodes (n' of Sec. 4.2) */
    uint64_t tests;              /* neighbours the projection test was evaluated for: the unseen ones; in long
                                    searches also already-seen ones that only the second level of the seen
                                    set would have recognised (it is consulted for passing neighbours only),
                                    unless PAG_FLAG_EXACT_TEST_COUNT is set */
    uint64_t passes;             /* of those, how many passed (gamma = passes / tests) */
    uint64_t exact;              /* exact distances computed, entry nodes included */
    uint64_t rounds;             /* TFB rounds */
    uint64_t rf_overflow;        /* entries overwritten in the ring R_F */
    uint64_t rt_overflow;        /* entries overwritten in the ring R_T */
    uint64_t seen_spills;        /* seen-set insertions that went to the HBM bitmap (all of them in long searches) */
    double   last_search_kernel_ms; /* HIP-event time of the search kernel of the last pag_search */
    double   last_prepare_ms;       /* HIP-event time of rotation + projection tables of the last pag_search */
    double   last_build_ms;         /* wall time of the last pag_build / pag_insert */
    uint64_t phase_cycles[6];       /* diagnostic: per-phase clock ticks of the search kernel, summed over waves;
                                       all zero unless the library was compiled with -DPAG_PHASE_TIMERS */
    uint64_t relinked_batches;      /* insertion batches, since the index was created, that were found to crowd a
                                       region of their own and were linked a second time (see pag_insert) */
    double   last_build_phase_ms[4]; /* HIP-event times of the last pag_build / pag_insert, summed over its batches:
                                       [0] the search kernel in indexing mode, [1] candidate sort + RobustPrune,
                                       [2] pair sort + reverse edges and PES verification, [3] inference information */
} pag_counters;

/*
 * pag_build (Alg. 1, Step 1, batch-synchronous): creates an index over the n
 * vectors D (dev, float32 [n*d]).  D is normalised (PAG_COS), rotated by Q and
 * copied into the index.  *out receives the handle.  Node i is row i of D.  The
 * nodes are linked in batches drawn from a shuffle of the ids that
 * pag_params.seed fixes, so the order in which the rows arrive (sorted by
 * cluster, source or time) does not shape the graph; the first 1024 nodes of
 * that shuffle are the entry nodes.
 */
int pag_build(const float* D, uint64_t n, uint32_t d, const pag_params* params, pag_index** out);

/*
 * pag_search (Alg. 2): K approximate nearest neighbours of each of the nq
 * queries Q (dev, float32 [nq*d]).  efS is the paper's efS: the number of TFB
 * rounds is ceil(efS / b).  Outputs (dev): ids int64 [nq*K], dists float32
 * [nq*K], per query ascending by (dist, id).  dists holds squared Euclidean
 * distances for PAG_L2 and 1 - <q,x> (= ||q-x||^2 / 2 on unit vectors) for
 * PAG_IP / PAG_COS.  Slots beyond the number of nodes reached hold id -1,
 * dist +inf.
 */
int pag_search(const pag_index* ix, const float* Q, uint64_t nq, uint32_t K, uint32_t efS,
               int64_t* ids, float* dists);

/*
 * pag_search_static: pag_search for callers that cannot allocate device memory -- code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same results.  It calls
 * no hipMalloc, hipFree or other allocating routine: its workspaces (rotated queries, projection tables,
 * normalised copies, per-wave seen-set bitmaps) live in one 48 MB device array that is part of the library
 * and that every GPU the library runs on holds until the process ends (its address on a GPU is looked up
 * when an index is created there, so the call itself loads nothing either).  Limits (PAG_EUNSUPPORTED beyond
 * them, nothing is launched): nq * (d + 16 * S [+ d for PAG_COS]) <= 4,194,304 floats, where S is
 * num_subspaces rounded up to 16, 32 or 64; index capacity <= 4,194,304 vectors; working set b <= 128
 * (K <= 128).  With fewer bitmaps than the GPU could keep waves busy the call is slower than pag_search,
 * never different; it also takes the queries as numbered (see PAG_FLAG_KEEP_QUERY_ORDER).  All calls on one GPU share the array: calls that overlap in time on one GPU (from
 * any thread, on any index) race and must be serialised by the caller.  The call synchronises the
 * index's stream before it returns, like pag_search.
 */
int pag_search_static(const pag_index* ix, const float* Q, uint64_t nq, uint32_t K, uint32_t efS,
                      int64_t* ids, float* dists);

/*
 * pag_insert (online insertion, Sec. 4.1): appends the m vectors X (dev,
 * float32 [m*d]); they receive ids n .. n+m-1 and are linked in shuffled
 * batches like the vectors of pag_build.  The vectors of one batch do not see
 * each other while they are linked; a batch found to crowd a region of its
 * own (vectors inserted where the index has none yet) is therefore linked a
 * second time once its vectors are part of the graph.
 * PAG_ECAPACITY if n + m exceeds pag_params.capacity.
 * If the call fails half way (a HIP error, memory), the index keeps answering
 * searches over the n vectors it had, but some of their out-edges may already
 * point at the vectors that were being added: further pag_insert calls on it
 * are refused with PAG_EINVAL.
 */
int pag_insert(pag_index* ix, const float* X, uint64_t m);

/* Waits for the index's stream, releases everything the index owns.  NULL is accepted.  Free its searchers first. */
int pag_free(pag_index* ix);

/* Fills n, d, num_subspaces, max_degree, n_entry, metric of `out` (pointers untouched). */
int pag_describe(const pag_index* ix, pag_arrays* out);
/* Copies the index into the caller-allocated host arrays of `out` (sizes as reported by pag_describe). */
int pag_export(const pag_index* ix, pag_arrays* out);
/* Creates an index from host arrays (all of them required); params gives capacity, efC, search_b, seed, stream.
 * The graph is validated on the host: PAG_EINVAL for a neighbour or entry id >= n, a code above 15, a neighbour
 * listed twice by one node, or an entry id listed twice. */
int pag_import(const pag_arrays* in, const pag_params* params, pag_index** out);

/* Statistics summed over all searches since the last reset (set out->struct_size first), and the reset. */
int pag_get_counters(const pag_index* ix, pag_counters* out);
int pag_reset_counters(pag_index* ix);
/* Changes search-time settings of an existing index: working-set size (0 = max(10,K)) and the search-time
 * PAG_FLAG_* bits (PAG_FLAG_NO_PRT, PAG_FLAG_EXACT_TEST_COUNT, PAG_FLAG_KEEP_QUERY_ORDER); the bits fixed at build time stay. */
int pag_set_search_options(pag_index* ix, uint32_t search_b, uint32_t flags);
/* log2 of the slots of the per-query LDS seen-set table; 0 = choose from efS.  Small values exercise the HBM spill path. */
int pag_set_seen_capacity_log2(pag_index* ix, uint32_t log2_slots);

/*
 * Single steps of the search, exposed for kernel-level parity checks.
 *
 * pag_prepare_queries (Alg. 2, rotation step and projection-table step):
 *   q_rot (dev float32 [nq*d]) and tables (dev float32 [nq*P*16],
 *   tables[i][l][j] = <q_l, r_jl>) of the queries Q (dev).
 * pag_exact_distances (Alg. 2, exact-distance step):
 *   keys[i*m+j] = ||q_rot[i] - x[ids[i*m+j]]||^2 for already rotated queries;
 *   ids dev uint32 [nq*m] (each < n), keys dev float32 [nq*m].
 * pag_screen (Eq. 3 + Eq. 4 in estimate form): for query i expanding node
 *   u[i] at squared distance Du[i], est[i*deg+s] = Du + c_s - 2 a_s S_s for
 *   every neighbour slot s of u[i] (NaN for a free slot); a neighbour passes
 *   the test iff est < ||z_max - q||^2.  tables as produced above.
 * pag_edge_info (Sec. 3.1 / Appendix B): recomputes codes, a, c, e2 of every
 *   stored edge of nodes [node_begin, node_end) from the vectors; outputs are
 *   host arrays [(node_end-node_begin)*deg (*P)].
 * pag_insertion_candidates (Alg. 1, the search of one insertion; Eq. 5): what
 *   inserting each of the m vectors X (dev, float32 [m*d], raw like the input of
 *   pag_insert) into the index as it stands would start from, without changing
 *   the index: the list R_L (capacity efC, ascending by (dist, id)) and the PES
 *   buffer H(v) (capacity max_degree, ascending).  Outputs are host arrays:
 *   cand_ids / cand_keys [m*efC] with cand_count [m] valid entries per vector,
 *   pes_ids / pes_keys [m*max_degree] with pes_count [m]; keys are squared
 *   distances.  With PAG_FLAG_NO_PES the buffers come back empty.
 */
int pag_prepare_queries(const pag_index* ix, const float* Q, uint64_t nq, float* q_rot, float* tables);
int pag_exact_distances(const pag_index* ix, const float* q_rot, uint64_t nq, const uint32_t* ids,
                        uint32_t m, float* keys);
int pag_screen(const pag_index* ix, const float* tables, uint64_t nq, const uint32_t* u,
               const float* Du, float* est);
int pag_edge_info(const pag_index* ix, uint64_t node_begin, uint64_t node_end, uint8_t* codes,
                  float* a, float* c, float* e2);
int pag_insertion_candidates(const pag_index* ix, const float* X, uint64_t m, uint32_t* cand_ids,
                             float* cand_keys, uint32_t* cand_count, uint32_t* pes_ids, float* pes_keys,
                             uint32_t* pes_count);

/*
 * Diagnostic for the roofline (no step of the method): reads `rows` whole rows of the index's vector
 * store, in order (scattered = 0) or in a scattered permutation (scattered = 1), four rows in flight
 * per wavefront, and reports the achieved rate in GB/s.  This is what the exact-distance step of
 * Alg. 2 could reach on this GPU if it did nothing but fetch its vectors.
 * scattered = 2 reproduces the traffic of whole hops of a long search instead: per seven random rows
 * one random adjacency record, eight random reads and seven random bit-sets in a per-wave seen-set
 * bitmap (the index's own workspace, cleared again afterwards); the rate counts rows and records only,
 * like the algorithmic bytes of the search do.
 */
int pag_measure_row_reads(const pag_index* ix, uint64_t rows, int scattered, double* gb_per_s);

/*
 * Searchers: searching while the index grows (the online-insertion setting of Sec. 5.2, D6).
 * A searcher is a view of an index with its own workspaces, counters and stream (a hipStream_t;
 * pass one that does not synchronise with the index's stream, else the calls just take turns).
 * pag_searcher_search is pag_search on that view: it sees the nodes whose insertion had completed when
 * the call began (pag_insert publishes its nodes after its last kernel has finished); nodes being inserted
 * are invisible.  While an insertion rewrites the out-edges of older nodes, a search may read an edge's
 * neighbour id and its inference information from different moments; that can change which neighbours
 * are tested in that hop, never a reported id/distance pair, which always comes from the stored vectors.
 * Results are therefore valid but, during an insertion, not reproducible bit for bit.
 * One searcher serves one call at a time; any number of searchers may share an index.  Free the
 * searchers before the index.  search_b, flags and the seen-set option are read from the index at each call.
 * For callers that insert and query at the same time from different host threads.
 */
typedef struct pag_searcher pag_searcher;
int pag_searcher_create(const pag_index* ix, void* stream, pag_searcher** out);
int pag_searcher_search(pag_searcher* s, const float* Q, uint64_t nq, uint32_t K, uint32_t efS,
                        int64_t* ids, float* dists);
int pag_searcher_get_counters(const pag_searcher* s, pag_counters* out);
int pag_searcher_free(pag_searcher* s);

const char* pag_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* PAG_H */
