/*
 * jx_oracle.c -- plain, slow, obviously-correct CPU implementation of the
 * Vamana beamSearch / robustPrune / batch-insert / RaBitQ path.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It exists to define what the GPU library
 * must compute.  Only the test-suite, the smoke check and the benchmark's
 * "cpu_baseline" leg may call it.  It shares no code, header, table or helper
 * with the HIP library and is never a fallback for it.
 *
 * Conventions
 *   - distance is squared L2 everywhere (App. B: the square root is elided);
 *     uint8 data uses exact 64-bit integers, float data double accumulators;
 *   - every comparison of candidates uses the strict total order
 *     (distance, id): smaller distance first, ties to the smaller id
 *     (the paper never mentions ties; this is this build's reading);
 *   - adjacency is a fixed-degree table adj[N][R] of uint32 ids, rows filled
 *     from the left, unused slots = 0xFFFFFFFF (Sec. 3.1: at most R out-edges);
 *   - floating point that decides an integer (the alpha test of robustPrune,
 *     a quantised code, the ordering of estimated distances) is evaluated in
 *     float32 with a fixed operation order and no fused multiply-add, so the
 *     GPU can take the same decision bit for bit.  Compile with
 *     -ffp-contract=off.
 *
 * Parallelism: OpenMP over independent queries / independent vertices only.
 * There is no blocking, tiling or reordering inside any single computation.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>
#include <float.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_U8 0
#define ORC_F32 1
#define ORC_F16 2 /* IEEE binary16 storage (App. D: float datasets are stored as FP16); arithmetic in double */
#define ORC_NONE 0xFFFFFFFFu

#define ORC_CAND_FRONTIER 0
#define ORC_CAND_VISITED 1

#define ORC_FILTER_EXACT 0 /* Alg. 1: exact visited set             */
#define ORC_FILTER_NONE 1  /* Alg. 2: no filter, duplicates dropped */

#define ORC_RULE_MAXCOS 0 /* grid point of largest cosine with r (sweep) */
#define ORC_RULE_MAXABS 1 /* fixed scale from max |r_i|                  */

typedef struct {
    double d;
    uint32_t id;
} orc_key;

static int key_less(double da, uint32_t ia, double db, uint32_t ib) {
    if (da < db) return 1;
    if (da > db) return 0;
    return ia < ib;
}

static int key_cmp(const void *a, const void *b) {
    const orc_key *x = (const orc_key *)a, *y = (const orc_key *)b;
    if (key_less(x->d, x->id, y->d, y->id)) return -1;
    if (key_less(y->d, y->id, x->d, x->id)) return 1;
    return 0;
}

/* ------------------------------------------------------------------ */
/* Distances (App. B: squared Euclidean distance, no square root)     */
/* ------------------------------------------------------------------ */

int64_t orc_l2sq_u8(const uint8_t *a, const uint8_t *b, int d) {
    int64_t s = 0;
    for (int i = 0; i < d; i++) {
        int64_t t = (int64_t)a[i] - (int64_t)b[i];
        s += t * t;
    }
    return s;
}

double orc_l2sq_f32(const float *a, const float *b, int d) {
    double s = 0.0;
    for (int i = 0; i < d; i++) {
        double t = (double)a[i] - (double)b[i];
        s += t * t;
    }
    return s;
}

/* exact value of an IEEE binary16 number */
static double half_to_double(uint16_t h) {
    const int sign = h >> 15, ex = (h >> 10) & 31, man = h & 1023;
    double v;
    if (ex == 0)
        v = ldexp((double)man, -24);
    else if (ex == 31)
        v = man ? NAN : INFINITY;
    else
        v = ldexp((double)(man | 1024), ex - 25);
    return sign ? -v : v;
}

double orc_l2sq_f16(const uint16_t *a, const uint16_t *b, int d) {
    double s = 0.0;
    for (int i = 0; i < d; i++) {
        double t = half_to_double(a[i]) - half_to_double(b[i]);
        s += t * t;
    }
    return s;
}

static size_t esize(int dtype) { return dtype == ORC_U8 ? 1 : (dtype == ORC_F16 ? 2 : 4); }

static double elem(int dtype, const void *v, size_t i) {
    if (dtype == ORC_U8) return (double)((const uint8_t *)v)[i];
    if (dtype == ORC_F16) return half_to_double(((const uint16_t *)v)[i]);
    return (double)((const float *)v)[i];
}

static double l2sq(int dtype, const void *a, const void *b, int d) {
    if (dtype == ORC_U8) return (double)orc_l2sq_u8((const uint8_t *)a, (const uint8_t *)b, d);
    if (dtype == ORC_F16) return orc_l2sq_f16((const uint16_t *)a, (const uint16_t *)b, d);
    return orc_l2sq_f32((const float *)a, (const float *)b, d);
}

/* ------------------------------------------------------------------ */
/* Distance providers for beamSearch                                   */
/* ------------------------------------------------------------------ */

typedef struct orc_dist_ctx {
    int mode; /* 0 exact, 1 RaBitQ integer-query estimator */
    /* exact */
    int dtype, d;
    const void *base;
    const void *query;
    /* rabitq */
    int bits, qbits, code_bytes;
    const uint8_t *codes; /* [N][code_bytes] */
    const float *meta;    /* [N][2] = data_add, data_rescale */
    const uint8_t *qint;  /* [d] */
    float q_lo, q_delta, q_add, q_sumq;
} orc_dist_ctx;

/* Code packing for m in {1, 2, 4, 8} bits: coordinate i occupies bits [i*m, (i+1)*m) of the little-endian bit
 * string (m = 1: bit i%8 of byte i/8; m = 4: low nibble for even i, high nibble for odd i; m = 8: byte i). */
static int code_get(const uint8_t *code, int bits, int i) {
    const int per = 8 / bits; /* coordinates per byte */
    return (code[i / per] >> ((i % per) * bits)) & ((1 << bits) - 1);
}

static void code_set(uint8_t *code, int bits, int i, int u) {
    const int per = 8 / bits;
    code[i / per] |= (uint8_t)(u << ((i % per) * bits));
}

/* Sec. 5.1, integer-query form of the estimator.  <u,q'> is approximated by
 * delta*<u,q_int> + lo*sum(u) where <u,q_int> is an exact integer; the five
 * float operations that follow are done in float32 in this fixed order. */
float orc_rabitq_est_int(const uint8_t *code, int bits, int d, float data_add, float data_rescale,
                         const uint8_t *qint, float q_lo, float q_delta, float q_add, float q_sumq) {
    int64_t I = 0, S = 0;
    for (int i = 0; i < d; i++) {
        int u = code_get(code, bits, i);
        I += (int64_t)u * (int64_t)qint[i];
        S += u;
    }
    float t = (float)I * q_delta;
    float t2 = q_lo * (float)S;
    t = t + t2;
    t = t - q_sumq;
    float e = data_add + q_add;
    float p = data_rescale * t;
    e = e + p;
    return e;
}

static double ctx_dist(const orc_dist_ctx *c, uint32_t id) {
    if (c->mode == 0) {
        const char *v = (const char *)c->base + (size_t)id * c->d * esize(c->dtype);
        return l2sq(c->dtype, c->query, v, c->d);
    }
    const uint8_t *code = c->codes + (size_t)id * c->code_bytes;
    return (double)orc_rabitq_est_int(code, c->bits, c->d, c->meta[2 * (size_t)id], c->meta[2 * (size_t)id + 1],
                                      c->qint, c->q_lo, c->q_delta, c->q_add, c->q_sumq);
}

/* ------------------------------------------------------------------ */
/* Brute-force k nearest neighbours (plain definition)                 */
/* ------------------------------------------------------------------ */

void orc_bruteforce(const void *base, int dtype, int64_t n, int d, const void *queries, int64_t nq, int k,
                    uint32_t *out_ids, double *out_dist, int nthreads) {
    size_t vs = (size_t)d * esize(dtype);
#pragma omp parallel for schedule(dynamic, 4) num_threads(nthreads)
    for (int64_t qi = 0; qi < nq; qi++) {
        orc_key *all = (orc_key *)malloc(sizeof(orc_key) * (size_t)(n > 0 ? n : 1));
        const char *q = (const char *)queries + (size_t)qi * vs;
        for (int64_t i = 0; i < n; i++) {
            all[i].d = l2sq(dtype, q, (const char *)base + (size_t)i * vs, d);
            all[i].id = (uint32_t)i;
        }
        qsort(all, (size_t)n, sizeof(orc_key), key_cmp);
        for (int j = 0; j < k; j++) {
            if (j < n) {
                out_ids[qi * k + j] = all[j].id;
                out_dist[qi * k + j] = all[j].d;
            } else {
                out_ids[qi * k + j] = ORC_NONE;
                out_dist[qi * k + j] = INFINITY;
            }
        }
        free(all);
    }
}

/* ------------------------------------------------------------------ */
/* beamSearch  (Alg. 1 and Alg. 2)                                     */
/* ------------------------------------------------------------------ */

typedef struct {
    double d;
    uint32_t id;
    int expanded;
} orc_fent;

/*
 * One query.  F is kept sorted by (distance, id).
 *   filter == ORC_FILTER_EXACT : Alg. 1 -- a neighbour is skipped if it has
 *       ever been seen (exact set).
 *   filter == ORC_FILTER_NONE  : Alg. 2 -- every neighbour's distance is
 *       computed; an id that is already an entry of F is not inserted twice.
 * Outputs: F (at most L entries) and the expansion list V in expansion order.
 * seen: caller-provided zeroed bitmap of n bits for ORC_FILTER_EXACT (left
 * zeroed again on return); may be NULL for ORC_FILTER_NONE.
 */
static void beam_search_one(const uint32_t *adj, int R, int64_t n, const orc_dist_ctx *ctx, int L, uint32_t start,
                            int filter, uint8_t *seen, orc_fent *F /* cap L+R */, int *out_nF, orc_key *V, int V_cap,
                            int *out_nV, int64_t *hops, int64_t *evals) {
    int nF = 0, nV = 0;
    int64_t nh = 0, ne = 0;
    uint32_t *touched = NULL;
    int64_t ntouched = 0, touched_cap = 0;
    (void)n;

    F[0].d = ctx_dist(ctx, start);
    F[0].id = start;
    F[0].expanded = 0;
    nF = 1;
    ne++;
    if (filter == ORC_FILTER_EXACT) {
        seen[start >> 3] |= (uint8_t)(1u << (start & 7));
        touched_cap = 1024;
        touched = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)touched_cap);
        touched[ntouched++] = start;
    }
    for (;;) {
        /* closest unexpanded entry: F is sorted, so the first one */
        int ui = -1;
        for (int i = 0; i < nF; i++)
            if (!F[i].expanded) {
                ui = i;
                break;
            }
        if (ui < 0) break;
        F[ui].expanded = 1;
        uint32_t u = F[ui].id;
        if (V && nV < V_cap) {
            V[nV].d = F[ui].d;
            V[nV].id = u;
        }
        nV++;
        nh++;
        const uint32_t *row = adj + (size_t)u * R;
        for (int j = 0; j < R; j++) {
            uint32_t v = row[j];
            if (v == ORC_NONE) break; /* rows are filled from the left */
            if (filter == ORC_FILTER_EXACT) {
                if (seen[v >> 3] & (1u << (v & 7))) continue;
                seen[v >> 3] |= (uint8_t)(1u << (v & 7));
                if (ntouched == touched_cap) {
                    touched_cap *= 2;
                    touched = (uint32_t *)realloc(touched, sizeof(uint32_t) * (size_t)touched_cap);
                }
                touched[ntouched++] = v;
            }
            double dv = ctx_dist(ctx, v);
            ne++;
            if (filter == ORC_FILTER_NONE) {
                int dup = 0;
                for (int i = 0; i < nF; i++)
                    if (F[i].id == v) {
                        dup = 1;
                        break;
                    }
                if (dup) continue;
            }
            /* sorted insertion */
            int pos = nF;
            while (pos > 0 && key_less(dv, v, F[pos - 1].d, F[pos - 1].id)) {
                F[pos] = F[pos - 1];
                pos--;
            }
            F[pos].d = dv;
            F[pos].id = v;
            F[pos].expanded = 0;
            nF++;
        }
        if (nF > L) nF = L; /* drop the furthest entries */
    }
    if (filter == ORC_FILTER_EXACT) {
        for (int64_t i = 0; i < ntouched; i++) seen[touched[i] >> 3] = 0;
        free(touched);
    }
    *out_nF = nF;
    if (out_nV) *out_nV = nV;
    if (hops) *hops += nh;
    if (evals) *evals += ne;
}

/* Exact-distance beamSearch for one query on a caller-supplied graph.
 * out_F_ids/out_F_dist: L slots (unused = NONE / +inf).  V_*: V_cap slots. */
void orc_beam_search(const uint32_t *adj, int R, const void *base, int dtype, int64_t n, int d, const void *query,
                     int L, uint32_t start, int filter, uint32_t *out_F_ids, double *out_F_dist, int32_t *out_nF,
                     uint32_t *out_V_ids, double *out_V_dist, int32_t V_cap, int32_t *out_nV, int64_t *out_hops,
                     int64_t *out_evals) {
    orc_dist_ctx ctx;
    memset(&ctx, 0, sizeof ctx);
    ctx.mode = 0;
    ctx.dtype = dtype;
    ctx.d = d;
    ctx.base = base;
    ctx.query = query;
    orc_fent *F = (orc_fent *)malloc(sizeof(orc_fent) * (size_t)(L + R + 1));
    orc_key *V = V_cap > 0 ? (orc_key *)malloc(sizeof(orc_key) * (size_t)V_cap) : NULL;
    uint8_t *seen = (uint8_t *)calloc((size_t)(n / 8 + 1), 1);
    int nF = 0, nV = 0;
    int64_t h = 0, e = 0;
    beam_search_one(adj, R, n, &ctx, L, start, filter, seen, F, &nF, V, V_cap, &nV, &h, &e);
    for (int i = 0; i < L; i++) {
        out_F_ids[i] = i < nF ? F[i].id : ORC_NONE;
        out_F_dist[i] = i < nF ? F[i].d : INFINITY;
    }
    *out_nF = nF;
    if (out_nV) *out_nV = nV;
    for (int i = 0; i < V_cap && i < nV; i++) {
        out_V_ids[i] = V[i].id;
        out_V_dist[i] = V[i].d;
    }
    if (out_hops) *out_hops = h;
    if (out_evals) *out_evals = e;
    free(F);
    free(V);
    free(seen);
}

/* Sec. 4.6: a logically deleted vertex is still traversed but must not appear in
 * any output: drop the deleted entries of a frontier, keeping the order. */
static int drop_deleted(orc_fent *F, int nF, const uint8_t *deleted) {
    int w = 0;
    if (!deleted) return nF;
    for (int i = 0; i < nF; i++)
        if (!deleted[F[i].id]) F[w++] = F[i];
    return w;
}

/* ------------------------------------------------------------------ */
/* robustPrune (Alg. 3)                                                */
/* ------------------------------------------------------------------ */

/*
 * cand: candidate (distance to p, id) pairs in any order; p_id is removed if
 * present, duplicate ids are removed (first occurrence after sorting wins --
 * equal ids carry equal distances).  Output: at most R ids in selection order.
 * The discard test alpha*d(p*,p') <= d(p,p') is applied to squared distances
 * and evaluated in float32: (float)alpha * (float)d1 <= (float)d2.
 */
int orc_robust_prune(uint32_t p_id, const uint32_t *cand_ids, const double *cand_dist, int64_t ncand, const void *base,
                     int dtype, int d, int R, float alpha, uint32_t *out_ids) {
    size_t vs = (size_t)d * esize(dtype);
    orc_key *c = (orc_key *)malloc(sizeof(orc_key) * (size_t)(ncand > 0 ? ncand : 1));
    int64_t m = 0;
    for (int64_t i = 0; i < ncand; i++) {
        if (cand_ids[i] == p_id || cand_ids[i] == ORC_NONE) continue;
        c[m].d = cand_dist[i];
        c[m].id = cand_ids[i];
        m++;
    }
    qsort(c, (size_t)m, sizeof(orc_key), key_cmp);
    /* drop duplicate ids: the first occurrence in sorted order is kept */
    int64_t w = 0;
    for (int64_t i = 0; i < m; i++) {
        int dup = 0;
        for (int64_t j = 0; j < w; j++)
            if (c[j].id == c[i].id) {
                dup = 1;
                break;
            }
        if (!dup) c[w++] = c[i];
    }
    m = w;
    uint8_t *dead = (uint8_t *)calloc((size_t)(m > 0 ? m : 1), 1);
    int nout = 0;
    for (int64_t i = 0; i < m && nout < R; i++) {
        if (dead[i]) continue;
        /* c[i] is the closest remaining candidate p* */
        out_ids[nout++] = c[i].id;
        const char *ps = (const char *)base + (size_t)c[i].id * vs;
        for (int64_t j = i + 1; j < m; j++) {
            if (dead[j]) continue;
            double dss = l2sq(dtype, ps, (const char *)base + (size_t)c[j].id * vs, d);
            float lhs = alpha * (float)dss;
            if (lhs <= (float)c[j].d) dead[j] = 1;
        }
    }
    free(dead);
    free(c);
    return nout;
}

/* ------------------------------------------------------------------ */
/* Index: store + graph + batch insertion (Alg. 4 with Sec. 4.3/4.5)   */
/* ------------------------------------------------------------------ */

typedef struct orc_index {
    int d, dtype, R, L_build, cand_mode;
    float alpha;
    float batch_growth; /* an internal batch holds at most max(1, floor(batch_growth * #linked)) points */
    int64_t capacity, n;
    uint32_t entry;
    void *base;    /* [capacity][d] */
    uint32_t *adj; /* [capacity][R] */
    uint8_t *deleted; /* [capacity] 1 = logically deleted (Sec. 4.6) */
    int64_t n_deleted;
    /* RaBitQ state (Sec. 5.1) */
    int bits, qbits, rule, code_bytes;
    float *P;       /* [d][d] row-major */
    float *c;       /* [d] */
    uint8_t *codes; /* [capacity][code_bytes] */
    float *meta;    /* [capacity][2] */
} orc_index;

orc_index *orc_index_create(int d, int dtype, int R, int L_build, float alpha, int64_t capacity, int cand_mode,
                            float batch_growth) {
    orc_index *x = (orc_index *)calloc(1, sizeof(orc_index));
    x->d = d;
    x->dtype = dtype;
    x->R = R;
    x->L_build = L_build;
    x->alpha = alpha;
    x->capacity = capacity;
    x->cand_mode = cand_mode;
    x->batch_growth = batch_growth;
    x->n = 0;
    x->entry = ORC_NONE;
    x->base = malloc((size_t)capacity * d * esize(dtype) + 16);
    x->adj = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)capacity * R + 16);
    memset(x->adj, 0xFF, sizeof(uint32_t) * (size_t)capacity * R);
    x->deleted = (uint8_t *)calloc((size_t)capacity + 1, 1);
    return x;
}

void orc_index_destroy(orc_index *x) {
    if (!x) return;
    free(x->base);
    free(x->adj);
    free(x->deleted);
    free(x->P);
    free(x->c);
    free(x->codes);
    free(x->meta);
    free(x);
}

int64_t orc_index_size(const orc_index *x) { return x->n; }
uint32_t orc_index_entry(const orc_index *x) { return x->entry; }

void orc_index_get_graph(const orc_index *x, uint32_t *adj_out, uint32_t *deg_out) {
    memcpy(adj_out, x->adj, sizeof(uint32_t) * (size_t)x->n * x->R);
    for (int64_t i = 0; i < x->n; i++) {
        int g = 0;
        while (g < x->R && x->adj[(size_t)i * x->R + g] != ORC_NONE) g++;
        deg_out[i] = (uint32_t)g;
    }
}

/* Load vectors + a ready-made graph (used to search a graph built elsewhere). */
void orc_index_set_graph(orc_index *x, const void *vecs, int64_t n, const uint32_t *adj, uint32_t entry) {
    memcpy(x->base, vecs, (size_t)n * x->d * esize(x->dtype));
    memcpy(x->adj, adj, sizeof(uint32_t) * (size_t)n * x->R);
    x->n = n;
    x->entry = entry;
}

static int row_degree(const uint32_t *row, int R) {
    int g = 0;
    while (g < R && row[g] != ORC_NONE) g++;
    return g;
}

typedef struct {
    uint32_t target;
    double d;
    uint32_t src;
} orc_edge;

static int edge_cmp(const void *a, const void *b) {
    const orc_edge *x = (const orc_edge *)a, *y = (const orc_edge *)b;
    if (x->target != y->target) return x->target < y->target ? -1 : 1;
    if (x->d != y->d) return x->d < y->d ? -1 : 1;
    if (x->src != y->src) return x->src < y->src ? -1 : 1;
    return 0;
}

/*
 * One batch X = ids[0..B) (all already present in the vector store, none yet
 * in the graph), inserted against the snapshot of the graph as it stands:
 *   1. beamSearch(G, x, L_build, entry) for every x, graph read-only;
 *   2. candidates = final frontier (default) or expansion list;
 *   3. adj[x] = robustPrune(x, candidates);
 *   4. reverse edges (v <- x, d(x,v)) for v in adj[x] only;
 *   5. sort by (target, distance, source);
 *   6. per target v: append if the row still fits, else
 *      adj[v] = robustPrune(v, adj[v] U new(v)) with d(v,.) recomputed.
 */
static void insert_subbatch(orc_index *x, const uint32_t *ids, int64_t B, int nthreads) {
    const int R = x->R, L = x->L_build, d = x->d;
    const size_t vs = (size_t)d * esize(x->dtype);
    const int64_t nsnap = x->capacity; /* bitmap covers every possible id */
    /* Expansion-list mode (Alg. 4 step 2 prunes V, the output of Alg. 1): the list keeps the first
       min(512, 4 L rounded up to a power of two) expanded vertices in expansion order (a search expands about
       1.2 L to 1.5 L vertices; the bound fixes the buffer of the GPU implementation, which uses the same one). */
    int V_cap = 0;
    if (x->cand_mode == ORC_CAND_VISITED) {
        V_cap = 64;
        while (V_cap < 4 * L && V_cap < 512) V_cap *= 2;
    }
    uint32_t *newrows = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)B * R);
    memset(newrows, 0xFF, sizeof(uint32_t) * (size_t)B * R);
    orc_edge *edges = (orc_edge *)malloc(sizeof(orc_edge) * (size_t)B * R + 16);
    int32_t *nrow = (int32_t *)calloc((size_t)B, sizeof(int32_t));

#pragma omp parallel num_threads(nthreads)
    {
        orc_fent *F = (orc_fent *)malloc(sizeof(orc_fent) * (size_t)(L + R + 1));
        orc_key *V = V_cap ? (orc_key *)malloc(sizeof(orc_key) * (size_t)V_cap) : NULL;
        uint8_t *seen = (uint8_t *)calloc((size_t)(nsnap / 8 + 1), 1);
        uint32_t *cid = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(V_cap > L ? V_cap : L));
        double *cd = (double *)malloc(sizeof(double) * (size_t)(V_cap > L ? V_cap : L));
#pragma omp for schedule(dynamic, 16)
        for (int64_t b = 0; b < B; b++) {
            uint32_t id = ids[b];
            orc_dist_ctx ctx;
            memset(&ctx, 0, sizeof ctx);
            ctx.mode = 0;
            ctx.dtype = x->dtype;
            ctx.d = d;
            ctx.base = x->base;
            ctx.query = (const char *)x->base + (size_t)id * vs;
            int nF = 0, nV = 0;
            beam_search_one(x->adj, R, nsnap, &ctx, L, x->entry, ORC_FILTER_EXACT, seen, F, &nF, V, V_cap, &nV, NULL,
                            NULL);
            nF = drop_deleted(F, nF, x->deleted); /* new points never link to deleted vertices */
            int nc = 0;
            if (x->cand_mode == ORC_CAND_FRONTIER) {
                for (int i = 0; i < nF; i++) {
                    cid[nc] = F[i].id;
                    cd[nc] = F[i].d;
                    nc++;
                }
            } else {
                int m = nV < V_cap ? nV : V_cap;
                for (int i = 0; i < m; i++) {
                    if (x->deleted && x->deleted[V[i].id]) continue; /* Sec. 4.6: never an output, so never a neighbour */
                    cid[nc] = V[i].id;
                    cd[nc] = V[i].d;
                    nc++;
                }
            }
            nrow[b] = orc_robust_prune(id, cid, cd, nc, x->base, x->dtype, d, R, x->alpha, newrows + (size_t)b * R);
        }
        free(F);
        free(V);
        free(seen);
        free(cid);
        free(cd);
    }
    /* write the new rows, emit reverse edges */
    int64_t ne = 0;
    for (int64_t b = 0; b < B; b++) {
        uint32_t id = ids[b];
        memcpy(x->adj + (size_t)id * R, newrows + (size_t)b * R, sizeof(uint32_t) * (size_t)R);
        for (int j = 0; j < nrow[b]; j++) {
            uint32_t v = newrows[(size_t)b * R + j];
            edges[ne].target = v;
            edges[ne].src = id;
            edges[ne].d = l2sq(x->dtype, (const char *)x->base + (size_t)id * vs, (const char *)x->base + (size_t)v * vs, d);
            ne++;
        }
    }
    qsort(edges, (size_t)ne, sizeof(orc_edge), edge_cmp);
    /* segment heads */
    int64_t *seg = (int64_t *)malloc(sizeof(int64_t) * (size_t)(ne + 1));
    int64_t nseg = 0;
    for (int64_t i = 0; i < ne; i++)
        if (i == 0 || edges[i].target != edges[i - 1].target) seg[nseg++] = i;
    seg[nseg] = ne;
#pragma omp parallel for schedule(dynamic, 64) num_threads(nthreads)
    for (int64_t s = 0; s < nseg; s++) {
        int64_t lo = seg[s], hi = seg[s + 1];
        uint32_t v = edges[lo].target;
        uint32_t *row = x->adj + (size_t)v * R;
        int g = row_degree(row, R);
        /* ids already present in the row are not new */
        int64_t m = 0;
        uint32_t *nid = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(hi - lo + R));
        double *nd = (double *)malloc(sizeof(double) * (size_t)(hi - lo + R));
        for (int64_t i = lo; i < hi; i++) {
            int present = 0;
            for (int j = 0; j < g; j++)
                if (row[j] == edges[i].src) {
                    present = 1;
                    break;
                }
            if (present) continue;
            nid[m] = edges[i].src;
            nd[m] = edges[i].d;
            m++;
        }
        if (g + m <= R) {
            for (int64_t i = 0; i < m; i++) row[g + i] = nid[i];
        } else {
            const char *pv = (const char *)x->base + (size_t)v * vs;
            for (int j = 0; j < g; j++) {
                nid[m] = row[j];
                nd[m] = l2sq(x->dtype, pv, (const char *)x->base + (size_t)row[j] * vs, d);
                m++;
            }
            uint32_t tmp[4096];
            uint32_t *outr = R <= 4096 ? tmp : (uint32_t *)malloc(sizeof(uint32_t) * (size_t)R);
            int k = orc_robust_prune(v, nid, nd, m, x->base, x->dtype, d, R, x->alpha, outr);
            for (int j = 0; j < R; j++) row[j] = j < k ? outr[j] : ORC_NONE;
            if (outr != tmp) free(outr);
        }
        free(nid);
        free(nd);
    }
    free(seg);
    free(edges);
    free(newrows);
    free(nrow);
    x->n += B;
}

/*
 * Append n vectors (ids = [N, N+n) in the given order) and link them in.
 *
 * Entry point (the paper says only "medoid"): the point of the FIRST insert
 * call nearest, by (distance, id), to that call's coordinate-wise mean; the
 * mean is accumulated in double and rounded to the data type's float32 image
 * (uint8 data: the mean is kept in float and distances are taken in double
 * against the float mean).  It joins the graph first, alone, with an empty row.
 *
 * Sub-batch schedule (the paper is silent on how a stream that starts empty is
 * bootstrapped; Sec. 6.2 reports batches of 0.5 % to 32 % of the index as
 * working): the remaining ids of the call, in increasing order, are cut into
 * sub-batches of size min(remaining, max(1, floor(batch_growth * #linked))).
 */
static int64_t batch_cap(const orc_index *x, int64_t linked) {
    int64_t c = (int64_t)floor((double)x->batch_growth * (double)linked);
    return c < 1 ? 1 : c;
}

int orc_index_insert(orc_index *x, const void *vecs, int64_t n, int nthreads) {
    if (x->n + n > x->capacity) return -1;
    const int d = x->d;
    const size_t vs = (size_t)d * esize(x->dtype);
    int64_t first = x->n;
    memcpy((char *)x->base + (size_t)first * vs, vecs, (size_t)n * vs);
    uint32_t *ids = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(n > 0 ? n : 1));
    int64_t m = 0;
    if (x->n == 0 && n > 0) {
        double *mean = (double *)calloc((size_t)d, sizeof(double));
        for (int64_t i = 0; i < n; i++)
            for (int j = 0; j < d; j++)
                mean[j] += elem(x->dtype, vecs, (size_t)i * d + j);
        for (int j = 0; j < d; j++) mean[j] = (double)(float)(mean[j] / (double)n);
        double best = INFINITY;
        uint32_t bi = 0;
        for (int64_t i = 0; i < n; i++) {
            double s = 0.0;
            for (int j = 0; j < d; j++) {
                double v = elem(x->dtype, vecs, (size_t)i * d + j);
                double t = v - mean[j];
                s += t * t;
            }
            if (s < best) {
                best = s;
                bi = (uint32_t)i;
            }
        }
        free(mean);
        x->entry = bi;
        /* the entry point joins first, alone, with no edges */
        for (int64_t i = 0; i < n; i++)
            if ((uint32_t)i != bi) ids[m++] = (uint32_t)i;
        x->n = 0;
        /* linked count is tracked separately from x->n during the first call:
           ids are not contiguous until the call completes */
        int64_t linked = 1, pos = 0;
        while (pos < m) {
            int64_t B = m - pos;
            if (B > batch_cap(x, linked)) B = batch_cap(x, linked);
            insert_subbatch(x, ids + pos, B, nthreads);
            pos += B;
            linked += B;
        }
        x->n = n;
        free(ids);
        return 0;
    }
    for (int64_t i = 0; i < n; i++) ids[m++] = (uint32_t)(first + i);
    int64_t pos = 0;
    while (pos < m) {
        int64_t linked = x->n;
        int64_t B = m - pos;
        if (B > batch_cap(x, linked)) B = batch_cap(x, linked);
        insert_subbatch(x, ids + pos, B, nthreads); /* advances x->n by B */
        pos += B;
    }
    free(ids);
    return 0;
}

/* ------------------------------------------------------------------ */
/* Batch deletion (Sec. 4.6; the algorithm of FreshDiskANN)             */
/* ------------------------------------------------------------------ */

/* Mark: a lightweight in-place operation.  Unknown / repeated ids are ignored. */
void orc_index_delete(orc_index *x, const uint32_t *ids, int64_t n) {
    for (int64_t i = 0; i < n; i++)
        if ((int64_t)ids[i] < x->n && !x->deleted[ids[i]]) {
            x->deleted[ids[i]] = 1;
            x->n_deleted++;
        }
}

int64_t orc_index_deleted_count(const orc_index *x) { return x->n_deleted; }

/*
 * Consolidate: every live vertex v that points to a deleted vertex gets, in
 * place of each deleted neighbour u, all of u's out-neighbours; the candidate
 * set (live vertices only, v itself excluded) is pruned with robustPrune.  All
 * new rows are computed from the graph as it stood before the call.  Then the
 * rows of the deleted vertices are emptied (nothing points to them any more).
 * If the entry point is deleted, the live vertex nearest to it (distance, then
 * id) becomes the new entry point.  Ids are not reused or renumbered.
 */
void orc_index_consolidate(orc_index *x, int nthreads) {
    const int R = x->R, d = x->d;
    const size_t vs = (size_t)d * esize(x->dtype);
    const int64_t n = x->n;
    uint32_t *newadj = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)n * R + 16);
    memcpy(newadj, x->adj, sizeof(uint32_t) * (size_t)n * R);
#pragma omp parallel for schedule(dynamic, 64) num_threads(nthreads)
    for (int64_t v = 0; v < n; v++) {
        if (x->deleted[v]) continue;
        const uint32_t *row = x->adj + (size_t)v * R;
        int g = row_degree(row, R), hit = 0;
        for (int j = 0; j < g; j++) hit |= x->deleted[row[j]];
        if (!hit) continue;
        uint32_t *cid = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(R + R * R));
        double *cd = (double *)malloc(sizeof(double) * (size_t)(R + R * R));
        int m = 0;
        const char *pv = (const char *)x->base + (size_t)v * vs;
        for (int j = 0; j < g; j++) {
            uint32_t u = row[j];
            if (!x->deleted[u]) {
                cid[m++] = u;
            } else {
                const uint32_t *ru = x->adj + (size_t)u * R;
                int gu = row_degree(ru, R);
                for (int t = 0; t < gu; t++)
                    if (!x->deleted[ru[t]] && ru[t] != (uint32_t)v) cid[m++] = ru[t];
            }
        }
        for (int i = 0; i < m; i++) cd[i] = l2sq(x->dtype, pv, (const char *)x->base + (size_t)cid[i] * vs, d);
        uint32_t *out = newadj + (size_t)v * R;
        int k = orc_robust_prune((uint32_t)v, cid, cd, m, x->base, x->dtype, d, R, x->alpha, out);
        for (int j = k; j < R; j++) out[j] = ORC_NONE;
        free(cid);
        free(cd);
    }
    for (int64_t v = 0; v < n; v++)
        if (x->deleted[v]) memset(newadj + (size_t)v * R, 0xFF, sizeof(uint32_t) * (size_t)R);
    memcpy(x->adj, newadj, sizeof(uint32_t) * (size_t)n * R);
    free(newadj);
    if (x->entry != ORC_NONE && x->deleted[x->entry]) {
        const char *pe = (const char *)x->base + (size_t)x->entry * vs;
        double best = INFINITY;
        uint32_t bi = ORC_NONE;
        for (int64_t v = 0; v < n; v++) {
            if (x->deleted[v]) continue;
            double dv = l2sq(x->dtype, pe, (const char *)x->base + (size_t)v * vs, d);
            if (dv < best) {
                best = dv;
                bi = (uint32_t)v;
            }
        }
        x->entry = bi;
    }
}

/*
 * Compact (Sec. 4.6, third phase): physically remove the deleted vertices.  It
 * may only follow a consolidation: no live row may still name a deleted vertex
 * (returns -1 otherwise, changing nothing).  Live vertices keep their relative
 * order: new id = number of live vertices with a smaller old id, so every
 * (distance, id) comparison -- and with it every search -- is unchanged up to
 * this renaming.  Vectors, rows, codes and the entry point move along; the
 * marks are cleared.  old_to_new [n_old] (may be NULL) receives the renaming,
 * ORC_NONE for removed vertices.  Returns the new number of points.
 */
int64_t orc_index_compact(orc_index *x, uint32_t *old_to_new) {
    const int R = x->R;
    const size_t vs = (size_t)x->d * esize(x->dtype);
    const int64_t n = x->n;
    for (int64_t v = 0; v < n; v++) {
        if (x->deleted[v]) continue;
        const uint32_t *row = x->adj + (size_t)v * R;
        for (int j = 0; j < R && row[j] != ORC_NONE; j++)
            if (x->deleted[row[j]]) return -1;
    }
    uint32_t *map = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(n + 1));
    int64_t live = 0;
    for (int64_t v = 0; v < n; v++) map[v] = x->deleted[v] ? ORC_NONE : (uint32_t)live++;
    for (int64_t v = 0; v < n; v++) {
        if (x->deleted[v]) continue;
        const int64_t w = map[v]; /* w <= v: moving in increasing order never overwrites an unread source */
        memmove((char *)x->base + (size_t)w * vs, (const char *)x->base + (size_t)v * vs, vs);
        uint32_t *dst = x->adj + (size_t)w * R;
        const uint32_t *src = x->adj + (size_t)v * R;
        for (int j = 0; j < R; j++) dst[j] = src[j] == ORC_NONE ? ORC_NONE : map[src[j]];
        if (x->bits) {
            memmove(x->codes + (size_t)w * x->code_bytes, x->codes + (size_t)v * x->code_bytes, (size_t)x->code_bytes);
            x->meta[2 * w] = x->meta[2 * v];
            x->meta[2 * w + 1] = x->meta[2 * v + 1];
        }
    }
    memset(x->adj + (size_t)live * R, 0xFF, sizeof(uint32_t) * (size_t)(n - live) * R);
    memset(x->deleted, 0, (size_t)n);
    if (x->entry != ORC_NONE) x->entry = map[x->entry];
    if (old_to_new) memcpy(old_to_new, map, sizeof(uint32_t) * (size_t)n);
    free(map);
    x->n = live;
    x->n_deleted = 0;
    return live;
}

/* ------------------------------------------------------------------ */
/* RaBitQ (Sec. 5.1)                                                   */
/* ------------------------------------------------------------------ */

/* r = P (v - c), accumulated in double, returned as float32 (the precision
 * in which every later code decision is taken) and optionally as double. */
void orc_rabitq_rotate(const float *vecs, int64_t n, int d, const float *P, const float *c, float *out_f32,
                       double *out_f64, int nthreads) {
#pragma omp parallel for schedule(static) num_threads(nthreads)
    for (int64_t i = 0; i < n; i++) {
        const float *v = vecs + (size_t)i * d;
        for (int a = 0; a < d; a++) {
            const float *row = P + (size_t)a * d;
            double s = 0.0;
            for (int b = 0; b < d; b++) s += (double)row[b] * ((double)v[b] - (double)c[b]);
            if (out_f32) out_f32[(size_t)i * d + a] = (float)s;
            if (out_f64) out_f64[(size_t)i * d + a] = s;
        }
    }
}

int orc_rabitq_code_bytes(int d, int bits) { return (d * bits + 7) / 8; }

typedef struct {
    double t;
    int i;
} orc_bp;

static int bp_cmp(const void *a, const void *b) {
    const orc_bp *x = (const orc_bp *)a, *y = (const orc_bp *)b;
    if (x->t < y->t) return -1;
    if (x->t > y->t) return 1;
    return x->i - y->i;
}

/*
 * Scale t of the m-bit grid for one rotated vector r (float32 values).
 * Grid vector xbar_i = sign(r_i) * (min(floor(t|r_i|), 2^(m-1)-1) + 1/2).
 *   MAXCOS: t maximises <xbar,r>/||xbar|| -- exact sweep over the breakpoints
 *           t = j/|r_i|, j = 1..2^(m-1)-1, with incremental updates of
 *           <xbar,|r|> and ||xbar||^2 in double; among equal cosines the
 *           smallest t wins.  The returned t is the breakpoint itself.
 *   MAXABS: t = (2^(m-1) - 1/2) / max|r_i|, computed in float32 as a single
 *           division, so that the largest coordinate lands mid-cell of the
 *           top level.
 * Returns t as a float (MAXABS) or double (MAXCOS) in *t_out; 0 if r == 0.
 */
static double grid_scale(const float *r, int d, int bits, int rule, double *cos_out) {
    const int half = 1 << (bits - 1); /* levels 0..half-1 */
    double amax = 0.0, l1 = 0.0, l2 = 0.0;
    for (int i = 0; i < d; i++) {
        double a = fabs((double)r[i]);
        if (a > amax) amax = a;
        l1 += a;
        l2 += a * a;
    }
    if (amax == 0.0) {
        if (cos_out) *cos_out = 0.0;
        return 0.0;
    }
    if (rule == ORC_RULE_MAXABS) {
        float t = ((float)half - 0.5f) / (float)amax;
        if (cos_out) {
            double ip = 0.0, nn = 0.0;
            for (int i = 0; i < d; i++) {
                float a = fabsf(r[i]);
                float lv = floorf(t * a);
                if (lv > (float)(half - 1)) lv = (float)(half - 1);
                double xb = (double)lv + 0.5;
                ip += xb * (double)a;
                nn += xb * xb;
            }
            *cos_out = ip / sqrt(nn) / sqrt(l2);
        }
        return (double)t;
    }
    /* sweep */
    int nb = 0;
    orc_bp *bp = (orc_bp *)malloc(sizeof(orc_bp) * (size_t)d * (size_t)(half > 1 ? half - 1 : 1));
    for (int i = 0; i < d; i++) {
        double a = fabs((double)r[i]);
        if (a == 0.0) continue;
        for (int j = 1; j < half; j++) {
            bp[nb].t = (double)j / a;
            bp[nb].i = i;
            nb++;
        }
    }
    qsort(bp, (size_t)nb, sizeof(orc_bp), bp_cmp);
    double ip = 0.5 * l1, nn = 0.25 * (double)d;
    double best = ip / sqrt(nn), best_t = 0.0;
    /* level of coordinate i after each breakpoint */
    int *lev = (int *)calloc((size_t)d, sizeof(int));
    int k = 0;
    while (k < nb) {
        double t = bp[k].t;
        /* apply every breakpoint that shares this t together */
        while (k < nb && bp[k].t == t) {
            int i = bp[k].i;
            lev[i]++;
            ip += fabs((double)r[i]);
            nn += 2.0 * (double)lev[i];
            k++;
        }
        double c = ip / sqrt(nn);
        if (c > best) {
            best = c;
            best_t = t;
        }
    }
    free(lev);
    free(bp);
    if (cos_out) *cos_out = best / sqrt(l2);
    return best_t;
}

/*
 * Encode n rotated vectors (float32 r = P(v-c)).
 *   code u_i in [0, 2^m): m = 1: u_i = [r_i >= 0];
 *   m > 1: level = min(floor(t*|r_i|), 2^(m-1)-1) with the scale t of
 *          grid_scale();  u_i = 2^(m-1) + level (r_i >= 0) or 2^(m-1)-1-level.
 *          For MAXCOS t is a breakpoint j/|r_k|: the level is then evaluated
 *          in double as floor(t*|r_i|) with the breakpoint's own coordinate
 *          landing exactly on j.  For MAXABS the product t*|r_i| is float32.
 *   xbar = u - (2^m - 1)/2.
 *   data_add = ||r||^2,  data_rescale = -2 ||r||^2 / <xbar, r>
 *   (both accumulated in double, stored as float32).  r == 0: code of the
 *   zero vector (all 2^(m-1), or all 1 for m = 1), data_add = data_rescale = 0.
 */
void orc_rabitq_encode(const float *r, int64_t n, int d, int bits, int rule, uint8_t *codes, float *meta,
                       double *cos_out, int nthreads) {
    const int cb = orc_rabitq_code_bytes(d, bits);
    const int half = 1 << (bits - 1);
    const double c_b = ((double)(1 << bits) - 1.0) / 2.0;
#pragma omp parallel for schedule(dynamic, 8) num_threads(nthreads)
    for (int64_t v = 0; v < n; v++) {
        const float *rv = r + (size_t)v * d;
        uint8_t *code = codes + (size_t)v * cb;
        memset(code, 0, (size_t)cb);
        double cosv = 0.0;
        double t = bits > 1 ? grid_scale(rv, d, bits, rule, &cosv) : 0.0;
        double l2 = 0.0, ip = 0.0;
        for (int i = 0; i < d; i++) {
            int u;
            double a = fabs((double)rv[i]);
            if (bits == 1) {
                u = rv[i] >= 0.0f ? 1 : 0;
            } else {
                int lv;
                if (rule == ORC_RULE_MAXABS) {
                    float p = (float)t * fabsf(rv[i]);
                    lv = (int)floorf(p);
                } else {
                    /* the level is the number of this coordinate's breakpoints
                       j/|r_i| (as computed by the sweep) that are <= t */
                    lv = 0;
                    if (a > 0.0)
                        while (lv + 1 < half && (double)(lv + 1) / a <= t) lv++;
                }
                if (lv > half - 1) lv = half - 1;
                if (lv < 0) lv = 0;
                u = rv[i] >= 0.0f ? half + lv : half - 1 - lv;
            }
            code_set(code, bits, i, u);
            l2 += a * a;
            ip += ((double)u - c_b) * (double)rv[i];
        }
        if (l2 == 0.0) {
            meta[2 * v] = 0.0f;
            meta[2 * v + 1] = 0.0f;
        } else {
            meta[2 * v] = (float)l2;
            meta[2 * v + 1] = (float)(-2.0 * l2 / ip);
        }
        if (cos_out) {
            if (bits == 1) {
                double l1 = 0.0;
                for (int i = 0; i < d; i++) l1 += fabs((double)rv[i]);
                cosv = l2 > 0 ? l1 / sqrt((double)d) / sqrt(l2) : 0.0;
            }
            cos_out[v] = cosv;
        }
    }
}

/*
 * Query record from a rotated query q' (float32):
 *   query_add  = ||q'||^2
 *   query_sumq = c_b * sum_i q'_i,  c_b = (2^m - 1)/2
 *   integer form with B_q bits: lo = min q', delta = (max q' - lo)/(2^B_q - 1),
 *   q_int_i = floor((q'_i - lo)/delta + 1/2) clamped to [0, 2^B_q - 1]
 *   (delta == 0: all zero).  lo, delta and the quotient are float32 operations
 *   in exactly this order; the two sums are accumulated in double.
 * out4 = {lo, delta, query_add, query_sumq}.
 */
void orc_rabitq_query_prep(const float *qr, int d, int bits, int qbits, uint8_t *qint, float *out4) {
    float lo = qr[0], hi = qr[0];
    double s = 0.0, s2 = 0.0;
    for (int i = 0; i < d; i++) {
        if (qr[i] < lo) lo = qr[i];
        if (qr[i] > hi) hi = qr[i];
        s += (double)qr[i];
        s2 += (double)qr[i] * (double)qr[i];
    }
    const float levels = (float)((1 << qbits) - 1);
    float delta = (hi - lo) / levels;
    for (int i = 0; i < d; i++) {
        int q = 0;
        if (delta > 0.0f) {
            float t = (qr[i] - lo) / delta;
            t = t + 0.5f;
            t = floorf(t);
            if (t < 0.0f) t = 0.0f;
            if (t > levels) t = levels;
            q = (int)t;
        }
        qint[i] = (uint8_t)q;
    }
    const double c_b = ((double)(1 << bits) - 1.0) / 2.0;
    out4[0] = lo;
    out4[1] = delta;
    out4[2] = (float)s2;
    out4[3] = (float)(c_b * s);
}

/* Float-query estimator in double: est = data_add + query_add
 *   + data_rescale * (<u,q'> - query_sumq).  Used only to pin the algebra. */
double orc_rabitq_est_float(const uint8_t *code, int bits, int d, double data_add, double data_rescale, const double *qr) {
    const double c_b = ((double)(1 << bits) - 1.0) / 2.0;
    double ip = 0.0, sq = 0.0, q2 = 0.0;
    for (int i = 0; i < d; i++) {
        ip += (double)code_get(code, bits, i) * qr[i];
        sq += qr[i];
        q2 += qr[i] * qr[i];
    }
    return data_add + q2 + data_rescale * (ip - c_b * sq);
}

/* exact integer inner product <u,q_int> and sum(u) (for the rounding-bound pin) */
void orc_rabitq_int_dot(const uint8_t *code, int bits, int d, const uint8_t *qint, int64_t *I, int64_t *S) {
    int64_t a = 0, b = 0;
    for (int i = 0; i < d; i++) {
        int u = code_get(code, bits, i);
        a += (int64_t)u * qint[i];
        b += u;
    }
    *I = a;
    *S = b;
}

void orc_rabitq_unpack(const uint8_t *code, int bits, int d, uint8_t *out) {
    for (int i = 0; i < d; i++) out[i] = (uint8_t)code_get(code, bits, i);
}

/*
 * Quantise the whole index (float32 data only).  centroid == NULL: mean of the
 * current base set, accumulated in double, rounded to float32, frozen.
 */
int orc_index_quantize(orc_index *x, int bits, int qbits, int rule, const float *P, const float *centroid,
                       int nthreads) {
    const int d = x->d;
    free(x->P);
    free(x->c);
    free(x->codes);
    free(x->meta);
    x->bits = bits;
    x->qbits = qbits;
    x->rule = rule;
    x->code_bytes = orc_rabitq_code_bytes(d, bits);
    x->P = (float *)malloc(sizeof(float) * (size_t)d * d);
    memcpy(x->P, P, sizeof(float) * (size_t)d * d);
    x->c = (float *)malloc(sizeof(float) * (size_t)d);
    if (centroid) {
        memcpy(x->c, centroid, sizeof(float) * (size_t)d);
    } else {
        double *m = (double *)calloc((size_t)d, sizeof(double));
        for (int64_t i = 0; i < x->n; i++)
            for (int j = 0; j < d; j++) m[j] += elem(x->dtype, x->base, (size_t)i * d + j);
        for (int j = 0; j < d; j++) x->c[j] = (float)(m[j] / (double)(x->n > 0 ? x->n : 1));
        free(m);
    }
    x->codes = (uint8_t *)malloc((size_t)x->capacity * x->code_bytes + 16);
    x->meta = (float *)malloc(sizeof(float) * 2 * (size_t)x->capacity + 16);
    float *r = (float *)malloc(sizeof(float) * (size_t)x->n * d + 16);
    const float *src = (const float *)x->base;
    float *tmp = NULL;
    if (x->dtype != ORC_F32) { /* binary16 -> float32 and uint8 -> float32 are exact */
        tmp = (float *)malloc(sizeof(float) * (size_t)x->n * d + 16);
        for (size_t i = 0; i < (size_t)x->n * d; i++) tmp[i] = (float)elem(x->dtype, x->base, i);
        src = tmp;
    }
    orc_rabitq_rotate(src, x->n, d, x->P, x->c, r, NULL, nthreads);
    free(tmp);
    orc_rabitq_encode(r, x->n, d, bits, rule, x->codes, x->meta, NULL, nthreads);
    free(r);
    return 0;
}

/* Install codes, the two floats per vector, rotation and centroid produced
 * elsewhere (used to time the estimator search on a large index whose codes
 * would take the plain double-precision rotation too long to recompute). */
void orc_index_set_codes(orc_index *x, int bits, int qbits, const float *P, const float *centroid, const uint8_t *codes,
                         const float *meta) {
    const int d = x->d;
    free(x->P);
    free(x->c);
    free(x->codes);
    free(x->meta);
    x->bits = bits;
    x->qbits = qbits;
    x->rule = ORC_RULE_MAXABS;
    x->code_bytes = orc_rabitq_code_bytes(d, bits);
    x->P = (float *)malloc(sizeof(float) * (size_t)d * d);
    memcpy(x->P, P, sizeof(float) * (size_t)d * d);
    x->c = (float *)malloc(sizeof(float) * (size_t)d);
    memcpy(x->c, centroid, sizeof(float) * (size_t)d);
    x->codes = (uint8_t *)malloc((size_t)x->capacity * x->code_bytes + 16);
    x->meta = (float *)malloc(sizeof(float) * 2 * (size_t)x->capacity + 16);
    memcpy(x->codes, codes, (size_t)x->n * x->code_bytes);
    memcpy(x->meta, meta, sizeof(float) * 2 * (size_t)x->n);
}

void orc_index_get_codes(const orc_index *x, uint8_t *codes, float *meta, float *centroid) {
    memcpy(codes, x->codes, (size_t)x->n * x->code_bytes);
    memcpy(meta, x->meta, sizeof(float) * 2 * (size_t)x->n);
    if (centroid) memcpy(centroid, x->c, sizeof(float) * (size_t)x->d);
}

/* ------------------------------------------------------------------ */
/* Search a batch of queries                                           */
/* ------------------------------------------------------------------ */

/*
 * mode 0: exact distances.  mode 1: RaBitQ integer-query estimator.
 * rerank == 0: the first k entries of F.  rerank > 0 (Sec. 5 / workload
 * definition): the first min(rerank, |F|) entries of F by (estimate, id) are
 * re-scored with the exact squared L2 (double) against the ORIGINAL query,
 * sorted by (distance, id), first k returned.
 * out_F_*: optional [nq][L] dump of the final frontier (ids, distances).
 * stats = {hops, dist_evals} summed over the batch.
 */
int orc_index_search(const orc_index *x, const void *queries, int64_t nq, int k, int L, int mode, int rerank, int filter,
                     uint32_t *out_ids, double *out_dist, uint32_t *out_F_ids, double *out_F_dist, int64_t *stats,
                     int nthreads) {
    if (k > L || x->n == 0) return -1;
    if (mode == 1 && !x->codes) return -2;
    const int d = x->d, R = x->R;
    const size_t vs = (size_t)d * esize(x->dtype);
    int64_t tot_h = 0, tot_e = 0;
#pragma omp parallel num_threads(nthreads) reduction(+ : tot_h, tot_e)
    {
        orc_fent *F = (orc_fent *)malloc(sizeof(orc_fent) * (size_t)(L + R + 1));
        uint8_t *seen = (uint8_t *)calloc((size_t)(x->capacity / 8 + 1), 1);
        float *qr = (float *)malloc(sizeof(float) * (size_t)d);
        uint8_t *qint = (uint8_t *)malloc((size_t)d);
        orc_key *rr = (orc_key *)malloc(sizeof(orc_key) * (size_t)(rerank > 0 ? rerank : 1));
#pragma omp for schedule(dynamic, 8)
        for (int64_t qi = 0; qi < nq; qi++) {
            const void *q = (const char *)queries + (size_t)qi * vs;
            orc_dist_ctx ctx;
            memset(&ctx, 0, sizeof ctx);
            ctx.dtype = x->dtype;
            ctx.d = d;
            ctx.base = x->base;
            ctx.query = q;
            if (mode == 1) {
                float m4[4];
                if (x->dtype != ORC_F32) {
                    float *qf = (float *)malloc(sizeof(float) * (size_t)d);
                    for (int j = 0; j < d; j++) qf[j] = (float)elem(x->dtype, q, (size_t)j);
                    orc_rabitq_rotate(qf, 1, d, x->P, x->c, qr, NULL, 1);
                    free(qf);
                } else {
                    orc_rabitq_rotate((const float *)q, 1, d, x->P, x->c, qr, NULL, 1);
                }
                orc_rabitq_query_prep(qr, d, x->bits, x->qbits, qint, m4);
                ctx.mode = 1;
                ctx.bits = x->bits;
                ctx.qbits = x->qbits;
                ctx.code_bytes = x->code_bytes;
                ctx.codes = x->codes;
                ctx.meta = x->meta;
                ctx.qint = qint;
                ctx.q_lo = m4[0];
                ctx.q_delta = m4[1];
                ctx.q_add = m4[2];
                ctx.q_sumq = m4[3];
            }
            int nF = 0;
            int64_t h = 0, e = 0;
            beam_search_one(x->adj, R, x->n, &ctx, L, x->entry, filter, seen, F, &nF, NULL, 0, NULL, &h, &e);
            nF = drop_deleted(F, nF, x->deleted);
            tot_h += h;
            tot_e += e;
            if (out_F_ids)
                for (int i = 0; i < L; i++) {
                    out_F_ids[qi * L + i] = i < nF ? F[i].id : ORC_NONE;
                    out_F_dist[qi * L + i] = i < nF ? F[i].d : INFINITY;
                }
            if (rerank > 0) {
                int m = nF < rerank ? nF : rerank;
                for (int i = 0; i < m; i++) {
                    rr[i].id = F[i].id;
                    rr[i].d = l2sq(x->dtype, q, (const char *)x->base + (size_t)F[i].id * vs, d);
                }
                qsort(rr, (size_t)m, sizeof(orc_key), key_cmp);
                for (int j = 0; j < k; j++) {
                    out_ids[qi * k + j] = j < m ? rr[j].id : ORC_NONE;
                    out_dist[qi * k + j] = j < m ? rr[j].d : INFINITY;
                }
            } else {
                for (int j = 0; j < k; j++) {
                    out_ids[qi * k + j] = j < nF ? F[j].id : ORC_NONE;
                    out_dist[qi * k + j] = j < nF ? F[j].d : INFINITY;
                }
            }
        }
        free(F);
        free(seen);
        free(qr);
        free(qint);
        free(rr);
    }
    if (stats) {
        stats[0] = tot_h;
        stats[1] = tot_e;
    }
    return 0;
}

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
