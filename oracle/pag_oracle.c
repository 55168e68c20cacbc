/*
 * pag_oracle.c -- plain CPU oracle for PAG (Projection-Augmented Graph) search.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement
 * of what the GPU library must compute.  It shares no code, header, table or
 * helper with the HIP path and is never called by it; only the tests, the
 * smoke check and the benchmark's CPU-baseline leg load it.
 *
 * Everything follows the paper's notation (u = node being expanded, w_i = its
 * out-neighbours, v or q = the point searched for, L subspaces -- called P
 * here, m = 16 projection vectors per subspace):
 *   - reference functions in fp64: Sec. 3.1 (cos alpha / beta / theta, Eq. 2),
 *     Eq. 3 (PRT), Eq. 4 (TFB threshold), Eq. 5 (PES), Appendix B (block-wise
 *     argmax that picks r*_il);
 *   - the search of Alg. 2 / Sec. 3.3 with the working set W, the rings R_F and
 *     R_T and the list R_L;
 *   - RobustPrune, Eq. 1 (alpha = 1), and Alg. 1: Step 1 per node, the PES screening of
 *     Step 2 and the verification of the buffered candidates (Step 3).
 *
 * Precision contract (decisions are taken in the same precision on both sides):
 *   rotated vectors, projection tables, exact distance keys and the stored
 *   per-edge scalars are fp64 sums of exact products, rounded once to fp32;
 *   the per-hop estimate is evaluated in fp32 as fmaf(-2 a_i, S_i, D_u + c_i)
 *   with S_i summed over the subspaces in increasing order.
 *
 * Parity pins: see tests/test_oracle_*.py.  One part is "parity unpinned":
 * which traversal the heuristic takes with the projection test active on
 * general data (the hop-synchronous reading below *is* the definition; what is
 * pinned are runs traced by hand -- the round mechanics with the test switched
 * off, the same with the test on where its estimate is exact (collinear
 * points, including an exact tie with the threshold), and one hop of a
 * hand-computed general case).  The pieces of Alg. 1 are pinned by hand-made
 * planar cases: the initial nodes, every branch of the reverse-edge rule, the
 * PES screening and the trimming of H(v) inside the search, the verification
 * of a buffered candidate, and one whole insertion traced by hand; the
 * batch-synchronous construction is pinned to the sequential one (batches of
 * one node give the same graph).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_EMPTY 0xFFFFFFFFu
#define ORC_M 16 /* projection vectors per subspace (Appendix D (1)) */

typedef struct {
    uint64_t n;        /* number of nodes */
    uint32_t d;        /* dimension */
    uint32_t P;        /* subspaces; dsub = d / P */
    uint32_t deg;      /* maximum out-degree (2M) */
    uint32_t n_entry;  /* entries in `entry` */
    float *vec;        /* [n*d] rotated base vectors */
    uint32_t *adj;     /* [n*deg] neighbour ids, ORC_EMPTY = free slot */
    float *a;          /* [n*deg] a_i = ||w_i-u|| / cos(beta_i) */
    float *c;          /* [n*deg] c_i = ||w_i-u||^2 + 2 a_i off_i */
    float *e2;         /* [n*deg] ||w_i-u||^2 */
    uint8_t *codes;    /* [n*deg*P] index of r*_il in codebook l (0..15) */
    const float *rot;  /* [d*d] orthogonal transform Q, row-major: q' = Q q */
    const float *cb;   /* [P*16*dsub] codebooks, vectors of norm 1/sqrt(P) */
    const uint32_t *entry; /* entry node ids */
} orc_index;

typedef struct {
    uint64_t queries, hops, tests, passes, exact, rounds, rf_over, rt_over;
} orc_counters;

/* ------------------------------------------------------------------ */
/* elementary pieces                                                   */
/* ------------------------------------------------------------------ */

/* squared Euclidean distance: differences taken in fp32, squares summed in fp64 */
double orc_sqdist64(uint32_t d, const float *x, const float *y) {
    double acc = 0.0;
    for (uint32_t k = 0; k < d; ++k) {
        float df = x[k] - y[k];
        acc += (double)df * (double)df;
    }
    return acc;
}

/* exact distance key used by the search (Alg. 2, exact-distance step) */
float orc_key(uint32_t d, const float *x, const float *y) {
    return (float)orc_sqdist64(d, x, y);
}

/* q' = Q q  (Alg. 2, rotation step) */
void orc_rotate(uint32_t d, const float *rot, const float *x, float *out) {
    for (uint32_t j = 0; j < d; ++j) {
        double acc = 0.0;
        for (uint32_t k = 0; k < d; ++k) acc += (double)rot[(uint64_t)j * d + k] * (double)x[k];
        out[j] = (float)acc;
    }
}

/* x / ||x||  (cosine: vectors are normalised, then ranked by Euclidean distance) */
void orc_normalise(uint32_t d, const float *x, float *out) {
    double s = 0.0;
    for (uint32_t k = 0; k < d; ++k) s += (double)x[k] * (double)x[k];
    double nrm = sqrt(s);
    if (nrm == 0.0) nrm = 1.0;
    for (uint32_t k = 0; k < d; ++k) out[k] = (float)((double)x[k] / nrm);
}

/* projection table T[l][j] = <q_l, r_jl>  (Alg. 2, projection-table step) */
void orc_table(uint32_t d, uint32_t P, const float *cb, const float *q, float *T, double *T64) {
    uint32_t ds = d / P;
    for (uint32_t l = 0; l < P; ++l)
        for (uint32_t j = 0; j < ORC_M; ++j) {
            const float *r = cb + ((uint64_t)l * ORC_M + j) * ds;
            double acc = 0.0;
            for (uint32_t k = 0; k < ds; ++k) acc += (double)r[k] * (double)q[l * ds + k];
            if (T) T[l * ORC_M + j] = (float)acc;
            if (T64) T64[l * ORC_M + j] = acc;
        }
}

/*
 * Inference information of one edge (u, w)  (Sec. 3.1; Appendix B, the argmax
 * that defines r*_il; Appendix C, what the structure I stores).
 *   codes[l] = argmax_j <r_jl, (w-u)_l>        (ties -> smallest j)
 *   out[0] = e2     = ||w-u||^2
 *   out[1] = maxsum = sum_l <r*_il, (w-u)_l>   (= ||w-u|| cos beta)
 *   out[2] = cosb   = maxsum / ||w-u||          (0 when w == u)
 *   out[3] = off    = sum_l <u_l, r*_il>
 *   out[4] = a      = ||w-u|| / max(cosb, 1e-6) (0 when w == u)
 *   out[5] = c      = e2 + 2 a off              (0 when w == u)
 */
void orc_edge_info(uint32_t d, uint32_t P, const float *cb, const float *u, const float *w,
                   uint8_t *codes, double *out) {
    uint32_t ds = d / P;
    double maxsum = 0.0, off = 0.0, e2 = 0.0;
    for (uint32_t l = 0; l < P; ++l) {
        double best = 0.0;
        uint32_t bj = 0;
        for (uint32_t j = 0; j < ORC_M; ++j) {
            const float *r = cb + ((uint64_t)l * ORC_M + j) * ds;
            double acc = 0.0;
            for (uint32_t k = 0; k < ds; ++k) {
                float df = w[l * ds + k] - u[l * ds + k];
                acc += (double)r[k] * (double)df;
            }
            if (j == 0 || acc > best) { best = acc; bj = j; }
        }
        const float *r = cb + ((uint64_t)l * ORC_M + bj) * ds;
        double o = 0.0;
        for (uint32_t k = 0; k < ds; ++k) o += (double)r[k] * (double)u[l * ds + k];
        codes[l] = (uint8_t)bj;
        maxsum += best;
        off += o;
    }
    for (uint32_t k = 0; k < d; ++k) {
        float df = w[k] - u[k];
        e2 += (double)df * (double)df;
    }
    double e = sqrt(e2);
    double cosb = 0.0, a = 0.0, c = 0.0;
    if (e2 > 0.0) {
        cosb = maxsum / e;
        double cb_clamped = cosb < 1e-6 ? 1e-6 : cosb;
        a = e / cb_clamped;
        c = e2 + 2.0 * a * off;
    }
    out[0] = e2; out[1] = maxsum; out[2] = cosb; out[3] = off; out[4] = a; out[5] = c;
}

/*
 * The statistics of Sec. 3 for one triple (u, w, v) written straight from their
 * definitions, in fp64, with square roots and divisions as printed:
 *   out[0] cos alpha  (Eq. 2)
 *   out[1] cos beta   (angle between r* and w-u)
 *   out[2] cos theta  (angle between r* and v-u; table lookup minus offset, over ||v-u||)
 *   out[3] tau        (Eq. 4) for the given squared distance dmax2 = ||z_max - v||^2
 *   out[4] PRT        (Eq. 3) = cos theta / cos beta - tau
 *   out[5] delta      (Sec. 3.4) = ||w-u|| / (2 ||v-u||)
 *   out[6] PES term   (Eq. 5)   = cos theta / cos beta - delta
 *   out[7] est        = D_u + c - 2 a S, the law-of-cosines estimate of ||v-w||^2
 *   out[8] S          = sum_l T_v[l][code_l]
 */
void orc_stats(uint32_t d, uint32_t P, const float *cb, const float *u, const float *w,
               const float *v, double dmax2, double *out) {
    uint32_t ds = d / P;
    uint8_t *codes = (uint8_t *)malloc(P);
    double info[6];
    orc_edge_info(d, P, cb, u, w, codes, info);
    double *T64 = (double *)malloc(sizeof(double) * P * ORC_M);
    orc_table(d, P, cb, v, NULL, T64);
    double S = 0.0;
    for (uint32_t l = 0; l < P; ++l) S += T64[l * ORC_M + codes[l]];
    double dot = 0.0, nw = 0.0, nv = 0.0;
    for (uint32_t k = 0; k < d; ++k) {
        double dw = (double)w[k] - (double)u[k], dv = (double)v[k] - (double)u[k];
        dot += dw * dv; nw += dw * dw; nv += dv * dv;
    }
    double ew = sqrt(nw), ev = sqrt(nv);
    /* r* is a unit vector (P blocks of norm 1/sqrt(P)), so <r*, x> / ||x|| is a cosine */
    double cos_alpha = dot / (ew * ev);
    double cos_beta = info[1] / ew;
    double cos_theta = (S - info[3]) / ev;
    double tau = (nw + nv - dmax2) / (2.0 * ev * ew);
    double delta = ew / (2.0 * ev);
    out[0] = cos_alpha; out[1] = cos_beta; out[2] = cos_theta; out[3] = tau;
    out[4] = cos_theta / cos_beta - tau;
    out[5] = delta;
    out[6] = cos_theta / cos_beta - delta;
    out[7] = nv + info[5] - 2.0 * info[4] * S;
    out[8] = S;
    (void)ds;
    free(T64); free(codes);
}

/* S_i = sum_l T[l][code_il], fp32, increasing l */
float orc_S32(uint32_t P, const float *T, const uint8_t *codes) {
    float S = 0.0f;
    for (uint32_t l = 0; l < P; ++l) S = S + T[l * ORC_M + codes[l]];
    return S;
}

/* est_i = D_u + c_i - 2 a_i S_i, fp32; PRT_i > 0  <=>  est_i < D_max (Eq. 3 + Eq. 4) */
float orc_est32(float Du, float a, float c, float S) {
    return fmaf(-2.0f * a, S, Du + c);
}

/* ------------------------------------------------------------------ */
/* search (Alg. 2, Sec. 3.3)                                            */
/* ------------------------------------------------------------------ */

typedef struct { float dist; uint32_t id; uint32_t visited; } ent;

static int ent_less(const ent *x, const ent *y) {
    return x->dist < y->dist || (x->dist == y->dist && x->id < y->id);
}
static int ent_cmp(const void *px, const void *py) {
    const ent *x = (const ent *)px, *y = (const ent *)py;
    if (ent_less(x, y)) return -1;
    if (ent_less(y, x)) return 1;
    return 0;
}

typedef struct { ent *e; uint32_t cap; uint64_t head; } ring; /* FIFO, overwrites the oldest */

static void ring_push(ring *r, ent x, uint64_t *over) {
    if (r->head >= r->cap) (*over)++;
    r->e[r->head % r->cap] = x;
    r->head++;
}
static uint32_t ring_count(const ring *r) { return r->head < r->cap ? (uint32_t)r->head : r->cap; }

enum { ORC_LITERAL = 1, ORC_NO_PRT = 2 };

typedef struct {
    uint8_t *seen;       /* n bytes, all zero between searches */
    uint32_t *seen_list; /* ids whose exact distance was computed, in order */
    uint64_t n_seen, cap_seen;
} orc_scratch;

static void scratch_mark(orc_scratch *s, uint32_t id) {
    if (s->n_seen == s->cap_seen) {
        s->cap_seen = s->cap_seen ? 2 * s->cap_seen : 1024;
        s->seen_list = (uint32_t *)realloc(s->seen_list, sizeof(uint32_t) * s->cap_seen);
    }
    s->seen[id] = 1;
    s->seen_list[s->n_seen++] = id;
}

/* one hop's admission step for a node whose exact distance is known (Alg. 2, inner if/else) */
static void admit(ent p, ent *W, uint32_t *nW, uint32_t b, ring *RF, ring *RT, orc_counters *ctr) {
    if (*nW < b) { W[(*nW)++] = p; return; }
    uint32_t worst = 0;
    for (uint32_t i = 1; i < *nW; ++i) if (ent_less(&W[worst], &W[i])) worst = i;
    if (ent_less(&p, &W[worst])) {
        ring_push(RT, W[worst], &ctr->rt_over); /* ejected z_max keeps its visited flag */
        W[worst] = p;
    } else {
        ring_push(RF, p, &ctr->rf_over);        /* false positive of the test */
    }
}

static float w_max(const ent *W, uint32_t nW, uint32_t b) {
    if (nW < b) return INFINITY;               /* z_max undefined: every unseen neighbour passes */
    float m = W[0].dist;
    for (uint32_t i = 1; i < nW; ++i) if (W[i].dist > m) m = W[i].dist;
    return m;
}

/*
 * PRT-TFB best-first search for one rotated query `q` with projection table T.
 *   b       working-set size; rounds R_max = ceil(ef / b)
 *   rl_cap  capacity of R_L (K when searching, efC when indexing)
 *   flags   0: hop-synchronous (threshold read once per expanded node, the hop's
 *              passers admitted in ascending (dist, id));
 *           ORC_LITERAL: threshold re-read before every single test, passers
 *              admitted one by one in stored neighbour order (Alg. 2 as printed);
 *           ORC_NO_PRT: the projection test is skipped (every unseen neighbour
 *              gets an exact distance).
 * n_nodes limits the graph to ids < n_nodes (used while indexing).
 * H (optional, indexing): PES candidate buffer of the searched point v (Alg. 1): every expanded
 * node u that survives the screening of Eq. 5 is recorded, the closest capH of them are kept,
 * ascending by (dist, id).
 * Output: out[0..*n_out) sorted by (dist, id).  scratch->seen is left cleared,
 * scratch->seen_list[0..n_seen) holds every node whose exact distance was computed.
 */
void orc_search_core(const orc_index *ix, uint64_t n_nodes, const float *q, const float *T,
                     uint32_t ef, uint32_t b, uint32_t rl_cap, int flags, orc_scratch *sc,
                     ent *out, uint32_t *n_out, orc_counters *ctr, ent *H, uint32_t *nH,
                     uint32_t capH) {
    const uint32_t d = ix->d, P = ix->P, deg = ix->deg;
    uint32_t Rmax = (ef + b - 1) / b;
    if (Rmax == 0) Rmax = 1;
    ent *W = (ent *)malloc(sizeof(ent) * b);
    ent *pass = (ent *)malloc(sizeof(ent) * deg);
    ent *RL = (ent *)malloc(sizeof(ent) * ((size_t)rl_cap + b));
    ent *merged = (ent *)malloc(sizeof(ent) * 2 * b);
    ring RF = { (ent *)malloc(sizeof(ent) * b), b, 0 };
    ring RT = { (ent *)malloc(sizeof(ent) * b), b, 0 };
    uint32_t nW = 0, nRL = 0;
    sc->n_seen = 0;
    ctr->queries++;

    /* b entry nodes with exact distances */
    for (uint32_t i = 0; i < ix->n_entry && nW < b; ++i) {
        uint32_t id = ix->entry[i];
        if (id >= n_nodes || sc->seen[id]) continue;
        ent e = { orc_key(d, q, ix->vec + (uint64_t)id * d), id, 0 };
        scratch_mark(sc, id);
        ctr->exact++;
        W[nW++] = e;
    }

    for (uint32_t r = 0; r < Rmax; ++r) {
        if (nW == 0) break;
        ctr->rounds++;
        for (;;) {
            /* closest unvisited node of W */
            int ui = -1;
            for (uint32_t i = 0; i < nW; ++i)
                if (!W[i].visited && (ui < 0 || ent_less(&W[i], &W[ui]))) ui = (int)i;
            if (ui < 0) break;
            W[ui].visited = 1;
            ctr->hops++;
            const uint32_t u = W[ui].id;
            const float Du = W[ui].dist;
            float Dmax = w_max(W, nW, b);
            uint32_t np = 0;
            if (H) {
                /* PES screening (Eq. 5): max_i (cos theta_i / cos beta_i - delta_i) < 0.  In estimate form
                 * (multiply through by 2 ||v-u|| ||w_i-u|| > 0): every est_i = D_u + c_i - 2 a_i S_i exceeds
                 * D_u, i.e. no out-neighbour of u is estimated to lie closer to v than u does. */
                int survives = 1;
                for (uint32_t i = 0; i < deg && survives; ++i) {
                    uint64_t s = (uint64_t)u * deg + i;
                    uint32_t w = ix->adj[s];
                    if (w == ORC_EMPTY || w >= n_nodes) continue;
                    float est = orc_est32(Du, ix->a[s], ix->c[s], orc_S32(P, T, ix->codes + s * P));
                    if (!(est > Du)) survives = 0;
                }
                if (survives) {
                    ent e = { Du, u, 0 };
                    uint32_t pos = *nH;
                    while (pos > 0 && ent_less(&e, &H[pos - 1])) pos--;
                    if (pos < capH) {
                        uint32_t last = *nH < capH ? *nH : capH - 1;
                        for (uint32_t k = last; k > pos; --k) H[k] = H[k - 1];
                        H[pos] = e;
                        if (*nH < capH) (*nH)++;
                    }
                }
            }
            for (uint32_t i = 0; i < deg; ++i) {
                uint64_t s = (uint64_t)u * deg + i;
                uint32_t w = ix->adj[s];
                if (w == ORC_EMPTY || w >= n_nodes || sc->seen[w]) continue;
                ctr->tests++;
                if (flags & ORC_LITERAL) Dmax = w_max(W, nW, b);
                int ok = 1;
                if (!(flags & ORC_NO_PRT)) {
                    float S = orc_S32(P, T, ix->codes + s * P);
                    float est = orc_est32(Du, ix->a[s], ix->c[s], S);
                    ok = est < Dmax;
                }
                if (!ok) continue;
                ent e = { orc_key(d, q, ix->vec + (uint64_t)w * d), w, 0 };
                scratch_mark(sc, w);
                ctr->passes++;
                ctr->exact++;
                if (flags & ORC_LITERAL) admit(e, W, &nW, b, &RF, &RT, ctr);
                else pass[np++] = e;
            }
            if (!(flags & ORC_LITERAL)) {
                qsort(pass, np, sizeof(ent), ent_cmp);
                for (uint32_t i = 0; i < np; ++i) admit(pass[i], W, &nW, b, &RF, &RT, ctr);
            }
        }
        /* round end: W -> R_L, clear W */
        for (uint32_t i = 0; i < nW; ++i) RL[nRL++] = W[i];
        qsort(RL, nRL, sizeof(ent), ent_cmp);
        if (nRL > rl_cap) nRL = rl_cap;
        nW = 0;
        /* merge and sort the rings, refill W, remainder back to R_T, clear R_F */
        uint32_t nm = 0;
        for (uint32_t i = 0; i < ring_count(&RF); ++i) merged[nm++] = RF.e[i];
        for (uint32_t i = 0; i < ring_count(&RT); ++i) merged[nm++] = RT.e[i];
        qsort(merged, nm, sizeof(ent), ent_cmp);
        RF.head = 0; RT.head = 0;
        for (uint32_t i = 0; i < nm && i < b; ++i) W[nW++] = merged[i];
        for (uint32_t i = nm; i > b; --i) ring_push(&RT, merged[i - 1], &ctr->rt_over); /* worst first */
    }
    for (uint32_t i = 0; i < nRL; ++i) out[i] = RL[i];
    *n_out = nRL;
    for (uint64_t i = 0; i < sc->n_seen; ++i) sc->seen[sc->seen_list[i]] = 0;
    free(W); free(pass); free(RL); free(merged); free(RF.e); free(RT.e);
}

/*
 * Batched search over raw (un-rotated) queries.  metric: 0 = L2 (keys are squared
 * distances), 1 = inner product on unit vectors, 2 = cosine (queries normalised
 * here); for 1 and 2 the reported key is ||q-x||^2 / 2 = 1 - <q,x>.
 * b = 0 selects max(10, K) (Alg. 2).  Unfilled slots: id -1, dist +inf.
 * seen_log (optional): per query, the list of seen ids is appended; seen_off[i]..seen_off[i+1].
 */
int orc_search_batch(const orc_index *ix, int metric, const float *Q, uint64_t nq, uint32_t K,
                     uint32_t efS, uint32_t b, int flags, int64_t *ids, float *dists,
                     orc_counters *ctr, uint32_t *seen_log, uint64_t seen_log_cap,
                     uint64_t *seen_off) {
    if (!ix || !Q || !ids || !dists || K == 0 || ix->d % ix->P != 0) return -1;
    const uint32_t d = ix->d, P = ix->P;
    if (b == 0) b = K > 10 ? K : 10;
    orc_scratch sc = { (uint8_t *)calloc(ix->n ? ix->n : 1, 1), NULL, 0, 0 };
    float *qn = (float *)malloc(sizeof(float) * d);
    float *qr = (float *)malloc(sizeof(float) * d);
    float *T = (float *)malloc(sizeof(float) * P * ORC_M);
    ent *out = (ent *)malloc(sizeof(ent) * ((size_t)K + b));
    orc_counters local;
    memset(&local, 0, sizeof local);
    uint64_t log_pos = 0;
    for (uint64_t i = 0; i < nq; ++i) {
        const float *q = Q + i * d;
        if (metric == 2) { orc_normalise(d, q, qn); q = qn; }
        orc_rotate(d, ix->rot, q, qr);
        orc_table(d, P, ix->cb, qr, T, NULL);
        uint32_t n_out = 0;
        orc_search_core(ix, ix->n, qr, T, efS, b, K, flags, &sc, out, &n_out, &local, NULL, NULL, 0);
        for (uint32_t k = 0; k < K; ++k) {
            if (k < n_out) {
                ids[i * K + k] = (int64_t)out[k].id;
                dists[i * K + k] = metric == 0 ? out[k].dist : 0.5f * out[k].dist;
            } else {
                ids[i * K + k] = -1;
                dists[i * K + k] = INFINITY;
            }
        }
        if (seen_off) {
            seen_off[i] = log_pos;
            for (uint64_t j = 0; j < sc.n_seen && seen_log && log_pos < seen_log_cap; ++j)
                seen_log[log_pos++] = sc.seen_list[j];
            seen_off[i + 1] = log_pos;
        }
    }
    if (ctr) {
        ctr->queries += local.queries; ctr->hops += local.hops; ctr->tests += local.tests;
        ctr->passes += local.passes; ctr->exact += local.exact; ctr->rounds += local.rounds;
        ctr->rf_over += local.rf_over; ctr->rt_over += local.rt_over;
    }
    free(sc.seen); free(sc.seen_list); free(qn); free(qr); free(T); free(out);
    return 0;
}

/* query preparation alone (rotation + table), for kernel-level parity tests */
int orc_prepare_queries(const orc_index *ix, int metric, const float *Q, uint64_t nq,
                        float *q_rot, float *tables) {
    const uint32_t d = ix->d, P = ix->P;
    float *qn = (float *)malloc(sizeof(float) * d);
    for (uint64_t i = 0; i < nq; ++i) {
        const float *q = Q + i * d;
        if (metric == 2) { orc_normalise(d, q, qn); q = qn; }
        orc_rotate(d, ix->rot, q, q_rot + i * d);
        orc_table(d, P, ix->cb, q_rot + i * d, tables + i * P * ORC_M, NULL);
    }
    free(qn);
    return 0;
}

/* ------------------------------------------------------------------ */
/* RobustPrune (Eq. 1, alpha = 1) and the per-node body of Alg. 1       */
/* ------------------------------------------------------------------ */

/*
 * Candidates sorted ascending by (distance to v, id).  A candidate c is kept
 * unless an already kept s has ||s-c|| <= ||v-c|| (then v can reach c through
 * s).  Stops at max_keep; no backfill.  Returns the number kept.
 */
static uint32_t robust_prune_of(const orc_index *ix, uint32_t self, uint32_t n_cand, const uint32_t *cand,
                                const float *cand_key, uint32_t max_keep, uint32_t *kept,
                                float *kept_key) {
    const uint32_t d = ix->d;
    uint32_t nk = 0;
    for (uint32_t i = 0; i < n_cand && nk < max_keep; ++i) {
        const float *cv = ix->vec + (uint64_t)cand[i] * d;
        int occluded = cand[i] == self;      /* a node that is in the graph already finds itself: never its own neighbour */
        for (uint32_t s = 0; s < nk && !occluded; ++s)
            if (orc_key(d, ix->vec + (uint64_t)kept[s] * d, cv) <= cand_key[i]) occluded = 1;
        if (!occluded) { kept[nk] = cand[i]; kept_key[nk] = cand_key[i]; nk++; }
    }
    return nk;
}

uint32_t orc_robust_prune(const orc_index *ix, uint32_t n_cand, const uint32_t *cand,
                          const float *cand_key, uint32_t max_keep, uint32_t *kept,
                          float *kept_key) {
    return robust_prune_of(ix, ORC_EMPTY, n_cand, cand, cand_key, max_keep, kept, kept_key);
}

static void write_edge(orc_index *ix, uint32_t u, uint32_t slot, uint32_t w) {
    uint64_t s = (uint64_t)u * ix->deg + slot;
    double info[6];
    ix->adj[s] = w;
    orc_edge_info(ix->d, ix->P, ix->cb, ix->vec + (uint64_t)u * ix->d, ix->vec + (uint64_t)w * ix->d,
                  ix->codes + s * ix->P, info);
    ix->e2[s] = (float)info[0];
    ix->a[s] = (float)info[4];
    ix->c[s] = (float)info[5];
}

static void clear_edge(orc_index *ix, uint32_t u, uint32_t slot) {
    uint64_t s = (uint64_t)u * ix->deg + slot;
    ix->adj[s] = ORC_EMPTY; ix->a[s] = 0; ix->c[s] = 0; ix->e2[s] = 0;
    memset(ix->codes + s * ix->P, 0, ix->P);
}

/*
 * Reverse edge u -> v after v chose u as an out-neighbour (Sec. 2.1, N_in(v)):
 * v is refused when some w in N_out(u) has ||w-v|| <= ||v-u|| and ||w-u|| <= ||v-u||
 * (Eq. 1).  Otherwise it takes a free slot; when u is full the list is re-pruned
 * incrementally: neighbours farther than v that v now occludes (||v-f|| <= ||f-u||)
 * are dropped, and if none is, the farthest of N_out(u) + {v} goes.
 */
void orc_reverse_edge(orc_index *ix, uint32_t u, uint32_t v, float duv) {
    const uint32_t d = ix->d, deg = ix->deg;
    const float *vv = ix->vec + (uint64_t)v * d;
    int free_slot = -1;
    uint32_t cnt = 0;
    for (uint32_t i = 0; i < deg; ++i) {
        uint64_t s = (uint64_t)u * deg + i;
        uint32_t w = ix->adj[s];
        if (w == ORC_EMPTY) { if (free_slot < 0) free_slot = (int)i; continue; }
        if (w == v) return;
        cnt++;
        if (ix->e2[s] <= duv && orc_key(d, ix->vec + (uint64_t)w * d, vv) <= duv) return;
    }
    if (cnt < deg) { write_edge(ix, u, (uint32_t)free_slot, v); return; }
    /* full list: who is farthest, and whom does v occlude? (nothing is modified in this pass) */
    const ent ev = { duv, v, 0 };
    int far = -1, n_occ = 0;
    ent efar = { 0, 0, 0 };
    uint8_t *occ = (uint8_t *)calloc(deg, 1);
    for (uint32_t i = 0; i < deg; ++i) {
        uint64_t s = (uint64_t)u * deg + i;
        ent ew = { ix->e2[s], ix->adj[s], 0 };
        if (far < 0 || ent_less(&efar, &ew)) { far = (int)i; efar = ew; }
        if (ent_less(&ev, &ew) && orc_key(d, ix->vec + (uint64_t)ew.id * d, vv) <= ew.dist) {
            occ[i] = 1; n_occ++;
        }
    }
    if (n_occ > 0) {
        int first = -1;
        for (uint32_t i = 0; i < deg; ++i)
            if (occ[i]) { clear_edge(ix, u, i); if (first < 0) first = (int)i; }
        write_edge(ix, u, (uint32_t)first, v);
    } else if (ent_less(&ev, &efar)) {
        write_edge(ix, u, (uint32_t)far, v);
    }
    free(occ);
}

/*
 * Verification of one PES candidate u -> v (Alg. 1, last loop): the RobustPrune condition of
 * Eq. 1 is evaluated exactly; an accepted edge is added only to a free out-degree slot of u,
 * existing edges are kept unchanged.  Returns 1 if the edge was added.
 */
int orc_pes_edge(orc_index *ix, uint32_t u, uint32_t v, float duv) {
    const uint32_t d = ix->d, deg = ix->deg;
    const float *vv = ix->vec + (uint64_t)v * d;
    int free_slot = -1;
    if (u == v) return 0;
    for (uint32_t i = 0; i < deg; ++i) {
        uint64_t s = (uint64_t)u * deg + i;
        uint32_t w = ix->adj[s];
        if (w == ORC_EMPTY) { if (free_slot < 0) free_slot = (int)i; continue; }
        if (w == v) return 0;
    }
    if (free_slot < 0) return 0;
    for (uint32_t i = 0; i < deg; ++i) {
        uint64_t s = (uint64_t)u * deg + i;
        uint32_t w = ix->adj[s];
        if (w == ORC_EMPTY) continue;
        if (ix->e2[s] <= duv && orc_key(d, ix->vec + (uint64_t)w * d, vv) <= duv) return 0;
    }
    write_edge(ix, u, (uint32_t)free_slot, v);
    return 1;
}

/*
 * The search of Alg. 1 for one point v (already rotated) over the nodes [0, n_nodes): Alg. 2's
 * loop with ef = efC, b = min(efC, 100) and R_L of capacity efC, plus the PES screening of every
 * expanded node.  Outputs R_L (ascending by (dist, id)) and the buffer H(v) (capacity deg = 2M,
 * ascending).  Exposed so that tests can look at the two lists themselves.
 */
int orc_index_search(const orc_index *ix, uint64_t n_nodes, const float *v, uint32_t efC,
                     uint32_t *cand_ids, float *cand_keys, uint32_t *n_cand,
                     uint32_t *pes_ids, float *pes_keys, uint32_t *n_pes, orc_counters *ctr) {
    const uint32_t d = ix->d, P = ix->P, deg = ix->deg;
    uint32_t b = efC < 100 ? efC : 100;
    if (b == 0 || d % P != 0) return -1;
    orc_counters local;
    memset(&local, 0, sizeof local);
    orc_scratch sc = { (uint8_t *)calloc(ix->n ? ix->n : 1, 1), NULL, 0, 0 };
    float *T = (float *)malloc(sizeof(float) * P * ORC_M);
    ent *rl = (ent *)malloc(sizeof(ent) * ((size_t)efC + b));
    ent *H = (ent *)malloc(sizeof(ent) * deg);
    uint32_t n_out = 0, nH = 0;
    orc_table(d, P, ix->cb, v, T, NULL);
    orc_search_core(ix, n_nodes, v, T, efC, b, efC, 0, &sc, rl, &n_out, &local, H, &nH, deg);
    for (uint32_t i = 0; i < n_out; ++i) { cand_ids[i] = rl[i].id; cand_keys[i] = rl[i].dist; }
    *n_cand = n_out;
    for (uint32_t i = 0; i < nH; ++i) { pes_ids[i] = H[i].id; pes_keys[i] = H[i].dist; }
    *n_pes = nH;
    if (ctr) *ctr = local;
    free(sc.seen); free(sc.seen_list); free(T); free(rl); free(H);
    return 0;
}

/* the first n_init nodes are linked to their nearest min(deg, n_init - 1) peers, ascending by (dist, id)
 * (Alg. 1: the initial nodes are selected and connected) */
static void init_nodes(orc_index *ix, uint64_t n_init) {
    const uint32_t d = ix->d, deg = ix->deg;
    ent *tmp = (ent *)malloc(sizeof(ent) * (n_init ? n_init : 1));
    for (uint64_t v = 0; v < n_init; ++v) {
        uint32_t m = 0;
        for (uint64_t o = 0; o < n_init; ++o) {
            if (o == v) continue;
            tmp[m].dist = orc_key(d, ix->vec + v * d, ix->vec + o * d);
            tmp[m].id = (uint32_t)o; tmp[m].visited = 0; m++;
        }
        qsort(tmp, m, sizeof(ent), ent_cmp);
        for (uint32_t i = 0; i < m && i < deg; ++i) write_edge(ix, (uint32_t)v, i, tmp[i].id);
    }
    free(tmp);
}

/*
 * Sequential construction (Alg. 1): nodes [n_start, n_end) are inserted one after another into
 * the graph that already holds nodes [0, n_start).  ix->vec must already hold the rotated
 * vectors of all nodes; adjacency arrays of the new nodes must be ORC_EMPTY.
 * With n_start == 0 the first min(efC, 100) nodes are the initial nodes: each is linked to its
 * nearest min(deg, .) among them.
 * Step 1 per node: search, RobustPrune -> N_out(v), reverse edges, inference information.
 * use_pes: Step 2 and Step 3 as well -- every insertion fills its buffer H(v) (capacity deg = 2M)
 * through the PES screening; the buffered candidates are verified after all insertions
 * (pes_every == 0, Alg. 1's last loop) or after every pes_every insertions (Sec. 4.2, online
 * insertion: the refinement runs after an insertion batch), in insertion order.
 */
int orc_build(orc_index *ix, uint32_t efC, uint64_t n_start, uint64_t n_end, orc_counters *ctr, int use_pes,
              uint64_t pes_every, uint64_t *pes_added) {
    const uint32_t d = ix->d, P = ix->P, deg = ix->deg;
    uint32_t b = efC < 100 ? efC : 100;
    if (b == 0 || d % P != 0) return -1;
    orc_counters local;
    memset(&local, 0, sizeof local);
    orc_scratch sc = { (uint8_t *)calloc(n_end ? n_end : 1, 1), NULL, 0, 0 };
    float *T = (float *)malloc(sizeof(float) * P * ORC_M);
    ent *rl = (ent *)malloc(sizeof(ent) * ((size_t)efC + b));
    uint32_t *cand = (uint32_t *)malloc(sizeof(uint32_t) * ((size_t)efC + b));
    float *ckey = (float *)malloc(sizeof(float) * ((size_t)efC + b));
    uint32_t *kept = (uint32_t *)malloc(sizeof(uint32_t) * deg);
    float *kkey = (float *)malloc(sizeof(float) * deg);
    const uint64_t count = n_end > n_start ? n_end - n_start : 0;
    ent *Hall = use_pes ? (ent *)malloc(sizeof(ent) * (size_t)(count ? count : 1) * deg) : NULL;
    uint32_t *nHall = use_pes ? (uint32_t *)calloc(count ? count : 1, sizeof(uint32_t)) : NULL;
    uint64_t v0 = n_start;
    if (n_start == 0) {
        uint64_t n_init = n_end < b ? n_end : b;
        init_nodes(ix, n_init);
        v0 = n_init;
    }
    uint64_t added = 0, verified = v0;     /* buffers of nodes [verified, v] are pending */
    for (uint64_t v = v0; v < n_end; ++v) {
        const float *vv = ix->vec + v * d;
        orc_table(d, P, ix->cb, vv, T, NULL);
        uint32_t n_out = 0;
        ent *H = use_pes ? Hall + (v - n_start) * deg : NULL;
        orc_search_core(ix, v, vv, T, efC, b, efC, 0, &sc, rl, &n_out, &local, H,
                        use_pes ? &nHall[v - n_start] : NULL, deg);
        for (uint32_t i = 0; i < n_out; ++i) { cand[i] = rl[i].id; ckey[i] = rl[i].dist; }
        uint32_t nk = orc_robust_prune(ix, n_out, cand, ckey, deg, kept, kkey);
        for (uint32_t i = 0; i < nk; ++i) write_edge(ix, (uint32_t)v, i, kept[i]);
        for (uint32_t i = 0; i < nk; ++i) orc_reverse_edge(ix, kept[i], (uint32_t)v, kkey[i]);
        const int flush = use_pes && (v + 1 == n_end || (pes_every && (v + 1 - v0) % pes_every == 0));
        if (flush) {
            for (uint64_t x = verified; x <= v; ++x) {
                const ent *Hx = Hall + (x - n_start) * deg;
                for (uint32_t i = 0; i < nHall[x - n_start]; ++i)
                    added += (uint64_t)orc_pes_edge(ix, Hx[i].id, (uint32_t)x, Hx[i].dist);
            }
            verified = v + 1;
        }
    }
    if (pes_added) *pes_added = added;
    if (ctr) *ctr = local;
    free(Hall); free(nHall);
    free(sc.seen); free(sc.seen_list); free(T); free(rl); free(cand); free(ckey); free(kept); free(kkey);
    return 0;
}

/*
 * Batch-synchronous construction: the reading of Alg. 1 for many insertions at once (the paper
 * builds with many threads and does not say in which order their updates land).  Nodes are taken
 * in id order in batches of m = min(remaining, max_batch, max(1, nodes in the graph / 2)).  The
 * nodes of a batch all search the graph as it was before the batch (they do not see each other);
 * then every one gets its N_out by RobustPrune; then the reverse edges and the buffered PES
 * candidates of the whole batch are applied target by target, for each target first the reverse
 * edges, then the PES candidates, each group ascending by distance (ties: by position of the
 * source in the batch, then by its slot).  With max_batch == 1 this is the sequential
 * construction with the PES buffers verified after every insertion.
 * What a sequential insertion has and a batch lacks is the sight of its batch-mates.  A batch found to
 * crowd a region of its own (batch_is_crowded below: vectors inserted where the graph has none yet) is
 * therefore linked a second time once its nodes are in the graph, in eight parts taken one after the other
 * (what one part links is there for the next): each node searches again (and finds itself, which RobustPrune
 * skips), its out-list is replaced by the new RobustPrune result, and the reverse edges and PES candidates
 * are applied as before.  relink == 0 leaves the second pass out (to show what
 * it is worth).
 */
typedef struct { uint32_t target, pes, src; float dist; uint64_t seq; } rev_pair;

static int pair_cmp(const void *px, const void *py) {
    const rev_pair *x = (const rev_pair *)px, *y = (const rev_pair *)py;
    if (x->target != y->target) return x->target < y->target ? -1 : 1;
    if (x->pes != y->pes) return x->pes < y->pes ? -1 : 1;
    if (x->dist != y->dist) return x->dist < y->dist ? -1 : 1;
    if (x->seq != y->seq) return x->seq < y->seq ? -1 : 1;
    return 0;
}

/*
 * Is a batch a region of its own?  (Batch-synchronous construction only; a sequential insertion sees
 * every earlier node and needs no such rule.)  For 128 nodes x of the batch [v0, v0 + m), spread evenly,
 * count among n_probe = min(m, v0, 2048) batch-mates and as many older nodes, both spread evenly, those
 * that lie closer to x than the farthest out-neighbour x has just been given.  In a batch that is mixed
 * like the graph the two counts agree; the batch is "crowded" when the mates number at least 32 and more
 * than four times the older nodes.
 */
static int batch_is_crowded(const orc_index *ix, uint64_t v0, uint64_t m) {
    const uint32_t d = ix->d, deg = ix->deg;
    const uint64_t n_sample = 128;
    uint64_t n_probe = m < v0 ? m : v0;
    if (n_probe > 2048) n_probe = 2048;
    uint64_t mates = 0, older = 0;
    for (uint64_t i = 0; i < n_sample; ++i) {
        const uint64_t x = v0 + i * m / n_sample;
        const float *xv = ix->vec + x * d;
        float far = 0.0f;
        for (uint32_t s = 0; s < deg; ++s)
            if (ix->adj[x * deg + s] != ORC_EMPTY && ix->e2[x * deg + s] > far) far = ix->e2[x * deg + s];
        for (uint64_t j = 0; j < n_probe; ++j) {
            const uint64_t y = v0 + j * m / n_probe, o = j * v0 / n_probe;
            if (y != x && orc_key(d, xv, ix->vec + y * d) < far) mates++;
            if (orc_key(d, xv, ix->vec + o * d) < far) older++;
        }
    }
    return mates >= 32 && (double)mates > 4.0 * (double)(older > 1 ? older : 1);
}

int orc_build_batched(orc_index *ix, uint32_t efC, uint64_t n_start, uint64_t n_end, uint64_t max_batch,
                      int use_pes, int relink, orc_counters *ctr, uint64_t *pes_added, uint64_t *n_batches,
                      uint64_t *n_relinked) {
    const uint32_t d = ix->d, P = ix->P, deg = ix->deg;
    uint32_t b = efC < 100 ? efC : 100;
    if (b == 0 || d % P != 0 || max_batch == 0) return -1;
    orc_counters local;
    memset(&local, 0, sizeof local);
    orc_scratch sc = { (uint8_t *)calloc(n_end ? n_end : 1, 1), NULL, 0, 0 };
    float *T = (float *)malloc(sizeof(float) * P * ORC_M);
    const size_t rl_room = (size_t)efC + b;
    ent *rl = (ent *)malloc(sizeof(ent) * rl_room * max_batch);      /* R_L of every node of the batch */
    uint32_t *n_rl = (uint32_t *)malloc(sizeof(uint32_t) * max_batch);
    ent *Hb = (ent *)malloc(sizeof(ent) * (size_t)deg * max_batch);  /* H(v) of every node of the batch */
    uint32_t *nHb = (uint32_t *)malloc(sizeof(uint32_t) * max_batch);
    uint32_t *cand = (uint32_t *)malloc(sizeof(uint32_t) * rl_room);
    float *ckey = (float *)malloc(sizeof(float) * rl_room);
    uint32_t *kept = (uint32_t *)malloc(sizeof(uint32_t) * deg);
    float *kkey = (float *)malloc(sizeof(float) * deg);
    rev_pair *pairs = (rev_pair *)malloc(sizeof(rev_pair) * 2 * (size_t)deg * max_batch);
    uint64_t v0 = n_start, added = 0, batches = 0, relinked = 0;
    if (n_start == 0) {
        uint64_t n_init = n_end < b ? n_end : b;
        init_nodes(ix, n_init);
        v0 = n_init;
    }
    while (v0 < n_end) {
        const uint64_t graph = v0;                       /* ids below v0 are in the graph */
        uint64_t m = n_end - v0;
        if (m > max_batch) m = max_batch;
        const uint64_t half = graph / 2 ? graph / 2 : 1;
        if (m > half) m = half;
        /* one linking pass over the batch; a crowded batch gets a second one, in which its nodes are part of the
         * graph, taken in eight parts one after the other (so that what one part links is there for the next) */
        const uint64_t parts = 8;
        for (uint64_t pass = 0; pass <= parts; ++pass) {
            const uint64_t visible = pass == 0 ? graph : graph + m;
            const uint64_t j0 = pass == 0 ? 0 : m * (pass - 1) / parts, j1 = pass == 0 ? m : m * pass / parts;
            /* 1. every node of the pass searches the graph as it is before the pass */
            for (uint64_t j = j0; j < j1; ++j) {
                const float *vv = ix->vec + (v0 + j) * d;
                orc_table(d, P, ix->cb, vv, T, NULL);
                nHb[j] = 0;
                orc_search_core(ix, visible, vv, T, efC, b, efC, 0, &sc, rl + j * rl_room, &n_rl[j], &local,
                                use_pes ? Hb + j * deg : NULL, use_pes ? &nHb[j] : NULL, deg);
            }
            /* 2. RobustPrune -> N_out(v), replacing what v had; the reverse edges and PES candidates are collected */
            uint64_t np = 0;
            for (int pes = 0; pes <= (use_pes ? 1 : 0); ++pes)
                for (uint64_t j = j0; j < j1; ++j) {
                    const uint32_t v = (uint32_t)(v0 + j);
                    if (!pes) {
                        const ent *r = rl + j * rl_room;
                        for (uint32_t i = 0; i < n_rl[j]; ++i) { cand[i] = r[i].id; ckey[i] = r[i].dist; }
                        uint32_t nk = robust_prune_of(ix, v, n_rl[j], cand, ckey, deg, kept, kkey);
                        for (uint32_t i = 0; i < deg; ++i) clear_edge(ix, v, i);
                        for (uint32_t i = 0; i < nk; ++i) {
                            write_edge(ix, v, i, kept[i]);
                            rev_pair p = { kept[i], 0, v, kkey[i], np };
                            pairs[np++] = p;
                        }
                    } else {
                        for (uint32_t i = 0; i < nHb[j]; ++i) {
                            const ent h = Hb[j * deg + i];
                            int dup = h.id == v;             /* already an out-neighbour of v: it has its reverse edge */
                            for (uint32_t s = 0; s < deg; ++s) if (ix->adj[(uint64_t)v * deg + s] == h.id) dup = 1;
                            if (dup) continue;
                            rev_pair p = { h.id, 1, v, h.dist, np };
                            pairs[np++] = p;
                        }
                    }
                }
            /* 3. applied target by target (an edge that exists already is left alone) */
            qsort(pairs, np, sizeof(rev_pair), pair_cmp);
            for (uint64_t i = 0; i < np; ++i) {
                if (pairs[i].pes) added += (uint64_t)orc_pes_edge(ix, pairs[i].target, pairs[i].src, pairs[i].dist);
                else orc_reverse_edge(ix, pairs[i].target, pairs[i].src, pairs[i].dist);
            }
            if (pass == 0) {
                if (!relink || m < 64 || graph < 64 || !batch_is_crowded(ix, v0, m)) break;
                relinked++;
            }
        }
        v0 += m;
        batches++;
    }
    if (pes_added) *pes_added = added;
    if (n_batches) *n_batches = batches;
    if (n_relinked) *n_relinked = relinked;
    if (ctr) *ctr = local;
    free(sc.seen); free(sc.seen_list); free(T); free(rl); free(n_rl); free(Hb); free(nHb);
    free(cand); free(ckey); free(kept); free(kkey); free(pairs);
    return 0;
}

/* recompute the inference information of every stored edge (used to check an imported index) */
int orc_edge_info_all(const orc_index *ix, uint64_t node_begin, uint64_t node_end, uint8_t *codes,
                      float *a, float *c, float *e2) {
    const uint32_t deg = ix->deg, P = ix->P, d = ix->d;
    double info[6];
    for (uint64_t u = node_begin; u < node_end; ++u)
        for (uint32_t i = 0; i < deg; ++i) {
            uint64_t s = u * deg + i, o = (u - node_begin) * deg + i;
            uint32_t w = ix->adj[s];
            if (w == ORC_EMPTY) { a[o] = 0; c[o] = 0; e2[o] = 0; memset(codes + o * P, 0, P); continue; }
            orc_edge_info(d, P, ix->cb, ix->vec + u * d, ix->vec + (uint64_t)w * d, codes + o * P, info);
            e2[o] = (float)info[0]; a[o] = (float)info[4]; c[o] = (float)info[5];
        }
    return 0;
}
