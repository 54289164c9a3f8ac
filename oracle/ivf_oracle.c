/*
 * CPU oracle for the IVF hot path -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Plain C, double-precision accumulation, no blocking, no intrinsics, no BLAS.
 * It shares nothing with the HIP library: no header, helper, table or layout.
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may use it.
 *
 * What it follows (paper sections, restated):
 *   - Section 2.2 ("Dynamic Vector Database"): an IVF index partitions the
 *     vectors into clusters; a query ranks the clusters by the distance from
 *     their centroids (coarse search), keeps the best nprobe of them and
 *     searches those clusters vector by vector (fine search).
 *   - Section 3.1 and the "IVF-Static" ablation of Section 6.1: a new vector is
 *     appended to the cluster of its nearest centroid; centroids never move and
 *     no other maintenance happens.
 *   - Section 4.4 ("CPU Insertion Buffer"): newly inserted vectors of a cluster
 *     are searched together with the cluster and the partial results merged,
 *     i.e. a search sees every vector inserted before it.
 *   - Section 3.2: one independent index per agent; a multi-agent search is a
 *     loop over the per-agent indexes.
 *
 * Readings where the paper is silent (kept identical in the design notes):
 *   one metric per index serves coarse ranking, assignment and fine search;
 *   L2 means the SQUARED Euclidean distance, computed as sum (q_i - x_i)^2;
 *   every tie goes to the lower id (results) / lower list number (centroids);
 *   rows shorter than k are padded with id -1 and +inf (L2) or -inf (IP);
 *   k-means is plain Lloyd under L2, initial centroids are rows chosen by the
 *   caller, an empty cluster keeps its previous centroid.
 *
 * Pins: see tests/test_oracle_pins.py (brute force against a matmul + lexsort,
 * nprobe = nlist equals brute force, insert-then-search self match, unit-norm
 * closed form L2 = 2 - 2 IP, nestedness in nprobe, partition invariants,
 * k-means monotone inertia and recovery of separated components, a hand-worked
 * 2-D example under tests/golden/).  No function here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_IP 0
#define ORC_L2 1

typedef struct {
    int64_t id;
    const float *vec; /* points into the caller's base array or into own[] */
} orc_entry;

typedef struct {
    orc_entry *e;
    int64_t len, cap;
} orc_list;

typedef struct orc_index {
    int d, nlist, metric;
    float *centroids; /* [nlist, d] private copy */
    orc_list *lists;
    /* inserted vectors are copied here in blocks so pointers stay valid */
    float **blocks;
    int64_t nblocks, block_fill, block_rows;
    int64_t ntotal, next_id;
} orc_index;

typedef struct {
    double v;
    int64_t id;
} orc_cand;

/* ---------------------------------------------------------------- scoring */

static double dot_d(const float *a, const float *b, int d)
{
    double s = 0.0;
    for (int i = 0; i < d; ++i) s += (double)a[i] * (double)b[i];
    return s;
}

static double l2sq_d(const float *a, const float *b, int d)
{
    double s = 0.0;
    for (int i = 0; i < d; ++i) {
        double t = (double)a[i] - (double)b[i];
        s += t * t;
    }
    return s;
}

/* value of a (query, vector) pair under the metric */
static double metric_value(int metric, const float *q, const float *x, int d)
{
    return metric == ORC_IP ? dot_d(q, x, d) : l2sq_d(q, x, d);
}

/* is (va, ida) strictly before (vb, idb) in result order? */
static int before(int metric, double va, int64_t ida, double vb, int64_t idb)
{
    if (va != vb) return metric == ORC_IP ? (va > vb) : (va < vb);
    return ida < idb;
}

static int g_sort_metric; /* qsort has no context argument; set under omp critical-free use: */
#pragma omp threadprivate(g_sort_metric)

static int cand_cmp(const void *pa, const void *pb)
{
    const orc_cand *a = (const orc_cand *)pa, *b = (const orc_cand *)pb;
    if (before(g_sort_metric, a->v, a->id, b->v, b->id)) return -1;
    if (before(g_sort_metric, b->v, b->id, a->v, a->id)) return 1;
    return 0;
}

static void sort_cands(int metric, orc_cand *c, int64_t n)
{
    g_sort_metric = metric;
    qsort(c, (size_t)n, sizeof(orc_cand), cand_cmp);
}

static void emit_topk(int metric, const orc_cand *c, int64_t n, int k, int64_t *ids, double *val)
{
    for (int j = 0; j < k; ++j) {
        if (j < n) {
            ids[j] = c[j].id;
            val[j] = c[j].v;
        } else {
            ids[j] = -1;
            val[j] = metric == ORC_IP ? -INFINITY : INFINITY;
        }
    }
}

/* best centroid for one vector: ties go to the lower list number */
static int nearest_centroid(const orc_index *ix, const float *x, double *best_out)
{
    int best = 0;
    double bv = metric_value(ix->metric, x, ix->centroids, ix->d);
    for (int j = 1; j < ix->nlist; ++j) {
        double v = metric_value(ix->metric, x, ix->centroids + (size_t)j * ix->d, ix->d);
        if (ix->metric == ORC_IP ? (v > bv) : (v < bv)) {
            bv = v;
            best = j;
        }
    }
    if (best_out) *best_out = bv;
    return best;
}

/* ------------------------------------------------------------------ index */

orc_index *orc_index_new(const float *centroids, int nlist, int d, int metric)
{
    if (!centroids || nlist < 1 || d < 1 || (metric != ORC_IP && metric != ORC_L2)) return NULL;
    orc_index *ix = (orc_index *)calloc(1, sizeof(orc_index));
    if (!ix) return NULL;
    ix->d = d;
    ix->nlist = nlist;
    ix->metric = metric;
    ix->centroids = (float *)malloc(sizeof(float) * (size_t)nlist * d);
    ix->lists = (orc_list *)calloc((size_t)nlist, sizeof(orc_list));
    ix->block_rows = 4096;
    if (!ix->centroids || !ix->lists) return NULL;
    memcpy(ix->centroids, centroids, sizeof(float) * (size_t)nlist * d);
    return ix;
}

void orc_index_free(orc_index *ix)
{
    if (!ix) return;
    for (int j = 0; j < ix->nlist; ++j) free(ix->lists[j].e);
    for (int64_t b = 0; b < ix->nblocks; ++b) free(ix->blocks[b]);
    free(ix->blocks);
    free(ix->lists);
    free(ix->centroids);
    free(ix);
}

static int list_push(orc_list *l, int64_t id, const float *vec)
{
    if (l->len == l->cap) {
        int64_t nc = l->cap ? l->cap * 2 : 16;
        orc_entry *ne = (orc_entry *)realloc(l->e, sizeof(orc_entry) * (size_t)nc);
        if (!ne) return -1;
        l->e = ne;
        l->cap = nc;
    }
    l->e[l->len].id = id;
    l->e[l->len].vec = vec;
    l->len++;
    return 0;
}

/* assignment only: list number of each row (Section 3.1 rule) */
int orc_assign(const orc_index *ix, const float *x, int64_t n, int32_t *lists_out)
{
    if (!ix || !x || !lists_out || n < 0) return -1;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < n; ++i)
        lists_out[i] = nearest_centroid(ix, x + (size_t)i * ix->d, NULL);
    return 0;
}

/*
 * Build: assign every base row to its best centroid and append it, in row
 * order.  The rows are NOT copied: `x` must outlive the index.  ids == NULL
 * numbers the rows from the index's running counter.
 */
int orc_build(orc_index *ix, const float *x, const int64_t *ids, int64_t n)
{
    if (!ix || (!x && n > 0) || n < 0) return -1;
    int32_t *a = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
    if (!a) return -1;
    orc_assign(ix, x, n, a);
    for (int64_t i = 0; i < n; ++i) {
        int64_t id = ids ? ids[i] : ix->next_id + i;
        if (list_push(&ix->lists[a[i]], id, x + (size_t)i * ix->d)) {
            free(a);
            return -1;
        }
    }
    if (!ids) ix->next_id += n;
    ix->ntotal += n;
    free(a);
    return 0;
}

static const float *own_copy(orc_index *ix, const float *x)
{
    if (ix->nblocks == 0 || ix->block_fill == ix->block_rows) {
        float **nb = (float **)realloc(ix->blocks, sizeof(float *) * (size_t)(ix->nblocks + 1));
        if (!nb) return NULL;
        ix->blocks = nb;
        ix->blocks[ix->nblocks] = (float *)malloc(sizeof(float) * (size_t)ix->block_rows * ix->d);
        if (!ix->blocks[ix->nblocks]) return NULL;
        ix->nblocks++;
        ix->block_fill = 0;
    }
    float *dst = ix->blocks[ix->nblocks - 1] + (size_t)ix->block_fill * ix->d;
    memcpy(dst, x, sizeof(float) * (size_t)ix->d);
    ix->block_fill++;
    return dst;
}

/*
 * Insert: the same nearest-centroid rule against the unchanged centroids,
 * appended at the tail of that list (vectors are copied).  forced_lists, when
 * given, overrides the rule (tests use it to mirror a legitimate near-tie flip).
 */
int orc_insert(orc_index *ix, const float *x, const int64_t *ids, int64_t m,
               const int32_t *forced_lists, int32_t *assigned_out)
{
    if (!ix || (!x && m > 0) || m < 0) return -1;
    for (int64_t i = 0; i < m; ++i) {
        const float *xi = x + (size_t)i * ix->d;
        int a = forced_lists ? forced_lists[i] : nearest_centroid(ix, xi, NULL);
        if (a < 0 || a >= ix->nlist) return -1;
        const float *kept = own_copy(ix, xi);
        if (!kept) return -1;
        int64_t id = ids ? ids[i] : ix->next_id + i;
        if (list_push(&ix->lists[a], id, kept)) return -1;
        if (assigned_out) assigned_out[i] = a;
    }
    if (!ids) ix->next_id += m;
    ix->ntotal += m;
    return 0;
}

/*
 * Delete (the interface of Section 5 has search, insert, delete and update): every stored
 * vector whose id is among ids[0..m) leaves its list, all of them if several carry the id;
 * the others keep their relative order.  Returns how many were removed, or -1.  An update
 * is a delete followed by an insert.
 */
int64_t orc_delete(orc_index *ix, const int64_t *ids, int64_t m)
{
    if (!ix || (!ids && m > 0) || m < 0) return -1;
    int64_t removed = 0;
    for (int j = 0; j < ix->nlist; ++j) {
        orc_list *L = &ix->lists[j];
        int64_t w = 0;
        for (int64_t r = 0; r < L->len; ++r) {
            int hit = 0;
            for (int64_t t = 0; t < m && !hit; ++t) hit = L->e[r].id == ids[t];
            if (hit) {
                ++removed;
            } else {
                L->e[w++] = L->e[r];
            }
        }
        L->len = w;
    }
    ix->ntotal -= removed;
    return removed;
}

/*
 * IVF-Split (Section 4.4 "on-GPU cluster splitting", Section 6.1 "Pancake-IVF-Split"): a
 * cluster that has grown past `threshold` vectors is split in two by a light k-means over
 * its members.  The paper gives no further rule; the reading taken here: lists are examined
 * in list order, only the lists that exist when the call starts; the two initial centroids
 * are the member with the smallest id and the member with the largest id (the first such
 * member in storage order if ids repeat); `iters` Lloyd iterations under L2 exactly as in
 * orc_kmeans (ties to the first of the two, a side without members keeps its centroid); the
 * members the last assignment put on the first side stay in the list, whose centroid
 * becomes the first centroid; the others form a new list appended after the last one, with
 * the second centroid.  Members keep their relative order.  Returns the number of splits.
 */
int orc_split(orc_index *ix, int64_t threshold, int iters)
{
    if (!ix || threshold < 1 || iters < 1) return -1;
    const int d = ix->d, nlist0 = ix->nlist;
    int nsplit = 0;
    for (int l = 0; l < nlist0; ++l) {
        orc_list *L = &ix->lists[l];
        const int64_t n = L->len;
        if (n <= threshold) continue;
        int64_t lo = 0, hi = 0;
        for (int64_t r = 1; r < n; ++r) {
            if (L->e[r].id < L->e[lo].id) lo = r;
            if (L->e[r].id > L->e[hi].id) hi = r;
        }
        double *c = (double *)malloc(sizeof(double) * 2 * d), *sum = (double *)malloc(sizeof(double) * 2 * d);
        int *a = (int *)malloc(sizeof(int) * (size_t)n);
        if (!c || !sum || !a) return -1;
        for (int t = 0; t < d; ++t) {
            c[t] = L->e[lo].vec[t];
            c[d + t] = L->e[hi].vec[t];
        }
        for (int it = 0; it < iters; ++it) {
            int64_t cnt[2] = {0, 0};
            memset(sum, 0, sizeof(double) * 2 * d);
            for (int64_t r = 0; r < n; ++r) {
                double s0 = 0.0, s1 = 0.0;
                for (int t = 0; t < d; ++t) {
                    double u0 = (double)L->e[r].vec[t] - c[t], u1 = (double)L->e[r].vec[t] - c[d + t];
                    s0 += u0 * u0;
                    s1 += u1 * u1;
                }
                a[r] = s1 < s0 ? 1 : 0;
                cnt[a[r]]++;
                for (int t = 0; t < d; ++t) sum[(size_t)a[r] * d + t] += L->e[r].vec[t];
            }
            for (int j = 0; j < 2; ++j)
                if (cnt[j] > 0)
                    for (int t = 0; t < d; ++t) c[(size_t)j * d + t] = sum[(size_t)j * d + t] / (double)cnt[j];
        }
        /* grow the tables by one list */
        float *nc = (float *)realloc(ix->centroids, sizeof(float) * (size_t)(ix->nlist + 1) * d);
        if (!nc) return -1;
        ix->centroids = nc;
        orc_list *nl = (orc_list *)realloc(ix->lists, sizeof(orc_list) * (size_t)(ix->nlist + 1));
        if (!nl) return -1;
        ix->lists = nl;
        L = &ix->lists[l];
        orc_list *N = &ix->lists[ix->nlist];
        memset(N, 0, sizeof(*N));
        for (int t = 0; t < d; ++t) {
            ix->centroids[(size_t)l * d + t] = (float)c[t];
            ix->centroids[(size_t)ix->nlist * d + t] = (float)c[d + t];
        }
        int64_t w = 0;
        for (int64_t r = 0; r < n; ++r) {
            if (a[r]) {
                if (list_push(N, L->e[r].id, L->e[r].vec)) return -1;
            } else {
                L->e[w++] = L->e[r];
            }
        }
        L->len = w;
        ix->nlist += 1;
        ++nsplit;
        free(c);
        free(sum);
        free(a);
    }
    return nsplit;
}

int orc_nlist(const orc_index *ix) { return ix ? ix->nlist : -1; }

int orc_centroids(const orc_index *ix, float *out)
{
    if (!ix || !out) return -1;
    memcpy(out, ix->centroids, sizeof(float) * (size_t)ix->nlist * ix->d);
    return 0;
}

int64_t orc_ntotal(const orc_index *ix) { return ix ? ix->ntotal : -1; }

int orc_list_lengths(const orc_index *ix, int64_t *len_out)
{
    if (!ix || !len_out) return -1;
    for (int j = 0; j < ix->nlist; ++j) len_out[j] = ix->lists[j].len;
    return 0;
}

/* ids of one list in storage order; returns the count written (<= cap) */
int64_t orc_list_ids(const orc_index *ix, int list, int64_t *ids_out, int64_t cap)
{
    if (!ix || list < 0 || list >= ix->nlist) return -1;
    int64_t n = ix->lists[list].len < cap ? ix->lists[list].len : cap;
    for (int64_t i = 0; i < n; ++i) ids_out[i] = ix->lists[list].e[i].id;
    return n;
}

/* ----------------------------------------------------------------- search */

/*
 * Coarse search (Section 2.2): score every centroid with the index metric,
 * keep the best nprobe, best first, ties to the lower list number.
 * scores_out (optional) receives all nlist scores per query.
 */
int orc_coarse(const orc_index *ix, const float *q, int64_t nq, int nprobe,
               int32_t *probes_out, double *scores_out)
{
    if (!ix || !q || !probes_out || nprobe < 1 || nprobe > ix->nlist) return -1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < nq; ++i) {
        orc_cand *c = (orc_cand *)malloc(sizeof(orc_cand) * (size_t)ix->nlist);
        for (int j = 0; j < ix->nlist; ++j) {
            c[j].v = metric_value(ix->metric, q + (size_t)i * ix->d,
                                  ix->centroids + (size_t)j * ix->d, ix->d);
            c[j].id = j;
            if (scores_out) scores_out[(size_t)i * ix->nlist + j] = c[j].v;
        }
        sort_cands(ix->metric, c, ix->nlist);
        for (int r = 0; r < nprobe; ++r) probes_out[(size_t)i * nprobe + r] = (int32_t)c[r].id;
        free(c);
    }
    return 0;
}

/*
 * Fine search over given probe lists (Section 2.2 fine search + Section 4.4
 * merge): every vector of every probed list, base rows and inserted rows
 * alike, is scored; candidates are ordered best-first with ties to the lower
 * id; the first k are returned, short rows padded.
 */
int orc_scan_probes(const orc_index *ix, const float *q, int64_t nq, int k, int nprobe,
                    const int32_t *probes, int64_t *ids_out, double *val_out)
{
    if (!ix || !q || !probes || k < 1 || nprobe < 1 || nprobe > ix->nlist) return -1;
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < nq; ++i) {
        const float *qi = q + (size_t)i * ix->d;
        int64_t total = 0;
        for (int r = 0; r < nprobe; ++r) {
            int l = probes[(size_t)i * nprobe + r];
            if (l < 0 || l >= ix->nlist) {
                bad = 1;
                l = 0;
            }
            total += ix->lists[l].len;
        }
        orc_cand *c = (orc_cand *)malloc(sizeof(orc_cand) * (size_t)(total > 0 ? total : 1));
        int64_t n = 0;
        for (int r = 0; r < nprobe; ++r) {
            int l = probes[(size_t)i * nprobe + r];
            if (l < 0 || l >= ix->nlist) continue;
            const orc_list *L = &ix->lists[l];
            for (int64_t t = 0; t < L->len; ++t) {
                c[n].v = metric_value(ix->metric, qi, L->e[t].vec, ix->d);
                c[n].id = L->e[t].id;
                ++n;
            }
        }
        sort_cands(ix->metric, c, n);
        emit_topk(ix->metric, c, n, k, ids_out + (size_t)i * k, val_out + (size_t)i * k);
        free(c);
    }
    return bad ? -1 : 0;
}

/* Coarse + fine search of one index (Section 2.2). */
int orc_search(const orc_index *ix, const float *q, int64_t nq, int k, int nprobe,
               int64_t *ids_out, double *val_out)
{
    if (!ix || !q || k < 1 || nprobe < 1 || nprobe > ix->nlist) return -1;
    int32_t *p = (int32_t *)malloc(sizeof(int32_t) * (size_t)(nq > 0 ? nq : 1) * nprobe);
    if (!p) return -1;
    int rc = orc_coarse(ix, q, nq, nprobe, p, NULL);
    if (!rc) rc = orc_scan_probes(ix, q, nq, k, nprobe, p, ids_out, val_out);
    free(p);
    return rc;
}

/*
 * Multi-agent search (Section 3.2, the per-agent-index scheme): query segment
 * a = rows [q_offsets[a], q_offsets[a+1]) is searched in handles[a]; no state
 * is shared between agents.
 */
int orc_search_multi(orc_index *const *handles, int n_handles, const int64_t *q_offsets,
                     const float *q, int k, int nprobe, int64_t *ids_out, double *val_out)
{
    if (!handles || !q_offsets || n_handles < 1) return -1;
    for (int a = 0; a < n_handles; ++a) {
        int64_t lo = q_offsets[a], hi = q_offsets[a + 1];
        if (hi < lo || !handles[a]) return -1;
        int rc = orc_search(handles[a], q + (size_t)lo * handles[a]->d, hi - lo, k, nprobe,
                            ids_out + (size_t)lo * k, val_out + (size_t)lo * k);
        if (rc) return rc;
    }
    return 0;
}

/*
 * Search over a scope of several memories (Section 3.2: every agent keeps its own
 * index, a request names the agents whose memories it may read, each of their indexes
 * is searched and the results are merged).  Every query is searched in every handle
 * (orc_scan_probes with that handle's probe lists, probes[h][i][r]); of the union of
 * the per-handle results the k best are returned, equal values ordered by the handle's
 * position in the scope, then by id.  src_out[i][j] is that position (-1 for padding).
 */
typedef struct {
    double v;
    int src;
    int64_t id;
} orc_ucand;

static int ucand_cmp(const void *pa, const void *pb)
{
    const orc_ucand *a = (const orc_ucand *)pa, *b = (const orc_ucand *)pb;
    if (a->v != b->v) {
        int a_first = g_sort_metric == ORC_IP ? (a->v > b->v) : (a->v < b->v);
        return a_first ? -1 : 1;
    }
    if (a->src != b->src) return a->src < b->src ? -1 : 1;
    if (a->id != b->id) return a->id < b->id ? -1 : 1;
    return 0;
}

int orc_union_probes(orc_index *const *handles, int n_handles, const float *q, int64_t nq, int k, int nprobe,
                     const int32_t *probes, int32_t *src_out, int64_t *ids_out, double *val_out)
{
    if (!handles || n_handles < 1 || !q || !probes || k < 1 || nq < 0) return -1;
    const int metric = handles[0]->metric, d = handles[0]->d;
    for (int h = 0; h < n_handles; ++h)
        if (!handles[h] || handles[h]->metric != metric || handles[h]->d != d) return -1;
    const size_t per = (size_t)(nq > 0 ? nq : 1) * k;
    int64_t *ids = (int64_t *)malloc(sizeof(int64_t) * per * n_handles);
    double *val = (double *)malloc(sizeof(double) * per * n_handles);
    if (!ids || !val) return -1;
    for (int h = 0; h < n_handles; ++h) {
        int rc = orc_scan_probes(handles[h], q, nq, k, nprobe, probes + (size_t)h * nq * nprobe, ids + per * h,
                                 val + per * h);
        if (rc) return rc;
    }
    orc_ucand *c = (orc_ucand *)malloc(sizeof(orc_ucand) * (size_t)n_handles * k);
    if (!c) return -1;
    for (int64_t i = 0; i < nq; ++i) {
        int64_t m = 0;
        for (int h = 0; h < n_handles; ++h)
            for (int j = 0; j < k; ++j) {
                const size_t at = per * h + (size_t)i * k + j;
                if (ids[at] < 0) continue; /* padding of a handle with fewer than k candidates */
                c[m].v = val[at];
                c[m].src = h;
                c[m].id = ids[at];
                ++m;
            }
        g_sort_metric = metric;
        qsort(c, (size_t)m, sizeof(orc_ucand), ucand_cmp);
        for (int j = 0; j < k; ++j) {
            const size_t at = (size_t)i * k + j;
            if (j < m) {
                src_out[at] = c[j].src;
                ids_out[at] = c[j].id;
                val_out[at] = c[j].v;
            } else {
                src_out[at] = -1;
                ids_out[at] = -1;
                val_out[at] = metric == ORC_IP ? -INFINITY : INFINITY;
            }
        }
    }
    free(c);
    free(ids);
    free(val);
    return 0;
}

/* the same with each handle's own coarse search (orc_coarse) */
int orc_search_union(orc_index *const *handles, int n_handles, const float *q, int64_t nq, int k, int nprobe,
                     int32_t *src_out, int64_t *ids_out, double *val_out)
{
    if (!handles || n_handles < 1 || nprobe < 1) return -1;
    int32_t *p = (int32_t *)malloc(sizeof(int32_t) * (size_t)n_handles * (nq > 0 ? nq : 1) * nprobe);
    if (!p) return -1;
    for (int h = 0; h < n_handles; ++h) {
        if (!handles[h] || nprobe > handles[h]->nlist) return -1;
        int rc = orc_coarse(handles[h], q, nq, nprobe, p + (size_t)h * nq * nprobe, NULL);
        if (rc) return rc;
    }
    int rc = orc_union_probes(handles, n_handles, q, nq, k, nprobe, p, src_out, ids_out, val_out);
    free(p);
    return rc;
}

/*
 * Exact k nearest neighbours over a raw array: what IVF approximates.  Does not
 * touch any index structure, so "nprobe = nlist equals brute force" compares
 * two separate code paths.
 */
int orc_bruteforce(const float *x, const int64_t *ids, int64_t n, int d, int metric,
                   const float *q, int64_t nq, int k, int64_t *ids_out, double *val_out)
{
    if ((!x && n > 0) || !q || k < 1 || d < 1 || (metric != ORC_IP && metric != ORC_L2)) return -1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < nq; ++i) {
        orc_cand *c = (orc_cand *)malloc(sizeof(orc_cand) * (size_t)(n > 0 ? n : 1));
        for (int64_t t = 0; t < n; ++t) {
            c[t].v = metric_value(metric, q + (size_t)i * d, x + (size_t)t * d, d);
            c[t].id = ids ? ids[t] : t;
        }
        sort_cands(metric, c, n);
        emit_topk(metric, c, n, k, ids_out + (size_t)i * k, val_out + (size_t)i * k);
        free(c);
    }
    return 0;
}

/* value of given (query row, vector row) pairs, one by one (full-size spot checks) */
int orc_pair_values(const float *q, const float *x, int64_t npairs, int d, int metric, double *val_out)
{
    if (!q || !x || !val_out) return -1;
    for (int64_t i = 0; i < npairs; ++i)
        val_out[i] = metric_value(metric, q + (size_t)i * d, x + (size_t)i * d, d);
    return 0;
}

/* ---------------------------------------------------------------- k-means */

/*
 * Lloyd's algorithm under L2.  init_rows[nlist] are the rows of x taken as the
 * initial centroids (the caller draws them from its seeded permutation).  Each
 * iteration assigns every row to its L2-nearest centroid (ties to the lower
 * index) and moves every non-empty centroid to the mean of its members; an
 * empty cluster keeps its centroid.  inertia_out[t] is the sum of squared
 * distances measured by the assignment step of iteration t.  Centroids are
 * kept in double during the run and rounded to float at the end.
 */
int orc_kmeans(const float *x, int64_t n, int d, int nlist, int iters, const int64_t *init_rows,
               float *centroids_out, double *inertia_out, int32_t *assign_out)
{
    if (!x || n < 1 || d < 1 || nlist < 1 || iters < 0 || !init_rows || !centroids_out) return -1;
    double *c = (double *)malloc(sizeof(double) * (size_t)nlist * d);
    double *sum = (double *)malloc(sizeof(double) * (size_t)nlist * d);
    int64_t *cnt = (int64_t *)malloc(sizeof(int64_t) * (size_t)nlist);
    int32_t *a = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    double *dist = (double *)malloc(sizeof(double) * (size_t)n);
    if (!c || !sum || !cnt || !a || !dist) return -1;
    for (int j = 0; j < nlist; ++j) {
        if (init_rows[j] < 0 || init_rows[j] >= n) return -1;
        for (int t = 0; t < d; ++t) c[(size_t)j * d + t] = x[(size_t)init_rows[j] * d + t];
    }
    for (int it = 0; it < iters; ++it) {
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < n; ++i) {
            const float *xi = x + (size_t)i * d;
            int best = 0;
            double bv = INFINITY;
            for (int j = 0; j < nlist; ++j) {
                const double *cj = c + (size_t)j * d;
                double s = 0.0;
                for (int t = 0; t < d; ++t) {
                    double u = (double)xi[t] - cj[t];
                    s += u * u;
                }
                if (s < bv) {
                    bv = s;
                    best = j;
                }
            }
            a[i] = best;
            dist[i] = bv;
        }
        double inertia = 0.0;
        memset(sum, 0, sizeof(double) * (size_t)nlist * d);
        memset(cnt, 0, sizeof(int64_t) * (size_t)nlist);
        for (int64_t i = 0; i < n; ++i) {
            inertia += dist[i];
            cnt[a[i]]++;
            for (int t = 0; t < d; ++t) sum[(size_t)a[i] * d + t] += x[(size_t)i * d + t];
        }
        if (inertia_out) inertia_out[it] = inertia;
        for (int j = 0; j < nlist; ++j)
            if (cnt[j] > 0)
                for (int t = 0; t < d; ++t) c[(size_t)j * d + t] = sum[(size_t)j * d + t] / (double)cnt[j];
    }
    for (size_t t = 0; t < (size_t)nlist * d; ++t) centroids_out[t] = (float)c[t];
    if (assign_out) memcpy(assign_out, a, sizeof(int32_t) * (size_t)n);
    free(c);
    free(sum);
    free(cnt);
    free(a);
    free(dist);
    return 0;
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
