/*
 * CPU oracle for the partition-local layer step of cache-assisted full-batch GNN training.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 definition of what the
 * HIP library must compute.  It shares no code, header, table or helper with the HIP
 * path and is never called by it.  Only the tests, the smoke check and the benchmark's
 * cpu_baseline leg may load it.
 *
 * Every floating-point routine works in double precision and sums each output element
 * sequentially in the order stated; OpenMP is used only across independent output
 * elements (rows, or feature columns), so results do not depend on the thread count.
 * The dense products of the combination step are not in this file: they are numpy's float64
 * matrix product, a library primitive, called from oracle.py.
 *
 * What each routine follows in the paper (arxiv 2508.13716):
 *   orc_placement     JACA, "Vertex Importance": cache the highest-priority halo vertices
 *                     first (Eq. 2 gives the priority; Alg. 1 "sort R(v_k) and select top k").
 *   orc_gather        JACA workflow: the receiving worker looks the halo rows up in the
 *                     local / global cache and places them in the layer input.
 *   orc_cache_update  "Vertex Importance and Vertex Update" / "Staleness in CaPGNN": cached rows are
 *                     overwritten with newer representations and carry the iteration they were written in.
 *   orc_stale_ids     bounded staleness: the rows that have not been refreshed for more than a
 *                     configured number of iterations.
 *   orc_influence     RAPA's vertex influence score (Eq. 6): degree-normalised sums over a vertex's outgoing
 *                     and incoming neighbours, times its repetition count.
 *   orc_locality_order  "we reorder the subgraphs" (end of the RAPA section, reorder figure): a new storage order
 *                     of the partition's vertices.  The paper names no algorithm; two orders are defined here.
 *   orc_gcn_scales    notation table: A-hat is the symmetrically normalised adjacency.
 *   orc_spmm_fwd      aggregation step of Eq. 1; A-hat * H in the GCN rule of Lemma 2's proof.
 *   orc_spmm_bwd      the transposed product the chain rule of that rule needs
 *                     (Lemma 3's recursion, operands put in conformable order).
 *   orc_softmax_ce    evaluation setup: cross-entropy loss for single-label tasks.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int orc_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void orc_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ---------------------------------------------------------------- placement (O1) */
typedef struct { int64_t prio, gid, idx; } orc_rank_t;

static int orc_rank_cmp(const void *a, const void *b)
{
    const orc_rank_t *x = (const orc_rank_t *)a, *y = (const orc_rank_t *)b;
    if (x->prio != y->prio) return (x->prio > y->prio) ? -1 : 1;   /* higher priority first */
    if (x->gid != y->gid) return (x->gid < y->gid) ? -1 : 1;       /* ties: smaller global id first */
    return 0;
}

/* order[k] = halo-local index of the k-th ranked vertex; tier[h] = 0 (GPU) for the first
 * min(cap_gpu, n_halo) ranked vertices, 1 (host) for the rest. */
void orc_placement(int64_t n_halo, const int64_t *gid, const int64_t *prio, int64_t cap_gpu,
                   int64_t *order, int8_t *tier)
{
    orc_rank_t *r = (orc_rank_t *)malloc(sizeof(orc_rank_t) * (size_t)(n_halo > 0 ? n_halo : 1));
    for (int64_t h = 0; h < n_halo; ++h) { r[h].prio = prio[h]; r[h].gid = gid[h]; r[h].idx = h; }
    qsort(r, (size_t)n_halo, sizeof(orc_rank_t), orc_rank_cmp);
    for (int64_t k = 0; k < n_halo; ++k) {
        order[k] = r[k].idx;
        tier[r[k].idx] = (k < cap_gpu) ? 0 : 1;
    }
    free(r);
}

/* ---------------------------------------------------------------- gather (O2) */
/* out[r, :] = table[ids[r], :] as raw bytes; an id outside [0, n_rows) gives a zero row.
 * Returns the number of such absent ids. */
int64_t orc_gather(const uint8_t *table, int64_t n_rows, int64_t row_bytes,
                   const int64_t *ids, int64_t n, uint8_t *out)
{
    int64_t absent = 0;
    for (int64_t r = 0; r < n; ++r) {
        int64_t id = ids[r];
        if (id < 0 || id >= n_rows) {
            memset(out + r * row_bytes, 0, (size_t)row_bytes);
            ++absent;
        } else {
            memcpy(out + r * row_bytes, table + id * row_bytes, (size_t)row_bytes);
        }
    }
    return absent;
}

/* table[ids[r], :] = rows[r, :] and stamp[ids[r]] = epoch, for r = 0..n-1 in this order (of several
 * updates of one row the last one stays); ids outside [0, n_rows) are skipped.  Returns how many were. */
int64_t orc_cache_update(uint8_t *table, int64_t *stamp, int64_t n_rows, int64_t row_bytes,
                         const int64_t *ids, int64_t n, const uint8_t *rows, int64_t epoch)
{
    int64_t absent = 0;
    for (int64_t r = 0; r < n; ++r) {
        int64_t id = ids[r];
        if (id < 0 || id >= n_rows) {
            ++absent;
            continue;
        }
        memcpy(table + id * row_bytes, rows + r * row_bytes, (size_t)row_bytes);
        stamp[id] = epoch;
    }
    return absent;
}

/* Rows whose stamp is more than max_age iterations behind epoch_now, in ascending order.
 * Returns their number; *oldest receives the smallest stamp (epoch_now if there are no rows). */
int64_t orc_stale_ids(const int64_t *stamp, int64_t n_rows, int64_t epoch_now, int64_t max_age,
                      int64_t *ids_out, int64_t *oldest)
{
    int64_t n = 0, lo = epoch_now;
    for (int64_t h = 0; h < n_rows; ++h) {
        if (stamp[h] < lo) lo = stamp[h];
        if (epoch_now - stamp[h] > max_age) ids_out[n++] = h;
    }
    *oldest = lo;
    return n;
}

/* Vertex influence score, Eq. 6, on a partition graph (rows = local vertices, entry (i, j) = edge j -> i):
 *   S_v = ( sum_{j in N_out(v)} 1/sqrt(Din_j) * 1/sqrt(Dout_v) + sum_{j in N_in(v)} 1/sqrt(Dout_j) * 1/sqrt(Din_v) ) * C_v
 * for every column vertex v (local vertices have both kinds of neighbours, halo vertices only outgoing ones).
 * din: in-degree of the local vertices [n_loc]; dout: out-degree of the column vertices [n_cols]; count: C [n_cols]. */
void orc_influence(int64_t n_loc, int64_t n_cols, const int64_t *rowptr, const int32_t *col,
                   const double *din, const double *dout, const double *count, double *S)
{
    for (int64_t v = 0; v < n_cols; ++v) S[v] = 0.0;
    /* outgoing neighbours of v: the rows i that hold an entry (i, v) */
    for (int64_t i = 0; i < n_loc; ++i)
        for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
            int64_t v = col[e];
            S[v] += (1.0 / sqrt(din[i])) * (1.0 / sqrt(dout[v]));
        }
    /* incoming neighbours of a local vertex i: the columns of its row */
    for (int64_t i = 0; i < n_loc; ++i)
        for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e)
            S[i] += (1.0 / sqrt(dout[col[e]])) * (1.0 / sqrt(din[i]));
    for (int64_t v = 0; v < n_cols; ++v) S[v] *= count[v];
}

/* ---------------------------------------------------------------- storage order of the vertices */
/* new2old[k] = the vertex stored at place k.  Local vertices keep places [0, n_loc), halo vertices the places
 * after them, so the partition keeps its shape and every result is the old one with rows permuted.
 *
 * method 0, by popularity: inside each of the two ranges, vertices referenced by more entries come first
 * (ties: smaller old index first).
 *
 * method 1, breadth first: local vertices in the order a breadth-first search over the local-to-local entries
 * reaches them.  A search starts at the unreached vertex with the longest row (ties: smaller index), a reached
 * vertex's row is scanned in stored order, and when a search dies out the next one starts the same way.
 * Halo vertices follow in the order in which the rows, walked in the new local order, first mention them;
 * halo vertices no row mentions come last, by index. */
typedef struct { int64_t key, idx; } orc_pair_t;

static int orc_pair_desc(const void *a, const void *b)
{
    const orc_pair_t *x = (const orc_pair_t *)a, *y = (const orc_pair_t *)b;
    if (x->key != y->key) return x->key > y->key ? -1 : 1;
    return x->idx < y->idx ? -1 : (x->idx > y->idx ? 1 : 0);
}

int orc_locality_order(int method, int64_t n_loc, int64_t n_halo, const int64_t *rowptr, const int32_t *col,
                       int32_t *new2old)
{
    const int64_t n_cols = n_loc + n_halo;
    orc_pair_t *byk = (orc_pair_t *)malloc((size_t)(n_cols > 0 ? n_cols : 1) * sizeof(orc_pair_t));
    char *seen = (char *)calloc((size_t)(n_cols > 0 ? n_cols : 1), 1);
    if (!byk || !seen) { free(byk); free(seen); return -1; }
    if (method == 0) {
        for (int64_t j = 0; j < n_cols; ++j) { byk[j].key = 0; byk[j].idx = j; }
        for (int64_t e = 0; e < rowptr[n_loc]; ++e) byk[col[e]].key += 1;
        qsort(byk, (size_t)n_loc, sizeof(orc_pair_t), orc_pair_desc);
        qsort(byk + n_loc, (size_t)n_halo, sizeof(orc_pair_t), orc_pair_desc);
        for (int64_t k = 0; k < n_cols; ++k) new2old[k] = (int32_t)byk[k].idx;
    } else {
        for (int64_t i = 0; i < n_loc; ++i) { byk[i].key = rowptr[i + 1] - rowptr[i]; byk[i].idx = i; }
        qsort(byk, (size_t)n_loc, sizeof(orc_pair_t), orc_pair_desc);
        int64_t placed = 0, head = 0;           /* new2old[0..placed) doubles as the search queue */
        for (int64_t s = 0; s < n_loc; ++s) {
            int64_t root = byk[s].idx;
            if (seen[root]) continue;
            seen[root] = 1;
            new2old[placed++] = (int32_t)root;
            while (head < placed) {
                int64_t u = new2old[head++];
                for (int64_t e = rowptr[u]; e < rowptr[u + 1]; ++e) {
                    int64_t v = col[e];
                    if (v < n_loc && !seen[v]) { seen[v] = 1; new2old[placed++] = (int32_t)v; }
                }
            }
        }
        for (int64_t k = 0; k < n_loc; ++k) {
            int64_t u = new2old[k];
            for (int64_t e = rowptr[u]; e < rowptr[u + 1]; ++e) {
                int64_t v = col[e];
                if (v >= n_loc && !seen[v]) { seen[v] = 1; new2old[placed++] = (int32_t)v; }
            }
        }
        for (int64_t v = n_loc; v < n_cols; ++v)
            if (!seen[v]) new2old[placed++] = (int32_t)v;
    }
    free(byk);
    free(seen);
    return 0;
}

/* ---------------------------------------------------------------- normalisation scales */
/* Symmetric normalisation A-hat[i,j] = r_i A_ij c_j with r_i = d_i^(-1/2), d_i = number of
 * stored entries of row i (the self loop is among them).  A local column j uses c_j = r_j; a
 * halo column uses its degree in the whole graph, clamped to at least 1. */
void orc_gcn_scales(int64_t n_loc, int64_t n_halo, const int64_t *rowptr,
                    const int64_t *halo_degree, double *r, double *c)
{
    for (int64_t i = 0; i < n_loc; ++i) {
        int64_t d = rowptr[i + 1] - rowptr[i];
        if (d < 1) d = 1;
        r[i] = 1.0 / sqrt((double)d);
        c[i] = r[i];
    }
    for (int64_t h = 0; h < n_halo; ++h) {
        int64_t d = halo_degree[h];
        if (d < 1) d = 1;
        c[n_loc + h] = 1.0 / sqrt((double)d);
    }
}

/* Mean aggregator: r_i = 1/deg_i (0 for an empty row), c_j = 1. */
void orc_mean_scales(int64_t n_loc, int64_t n_cols, const int64_t *rowptr, double *r, double *c)
{
    for (int64_t i = 0; i < n_loc; ++i) {
        int64_t d = rowptr[i + 1] - rowptr[i];
        r[i] = d > 0 ? 1.0 / (double)d : 0.0;
    }
    for (int64_t j = 0; j < n_cols; ++j) c[j] = 1.0;
}

/* ---------------------------------------------------------------- SpMM (O3, O4) */
/* Y[i,f] = r[i] * sum_{e in row i, in order} v[e] * c[col[e]] * X[col[e], f];  v == NULL means 1. */
void orc_spmm_fwd(int64_t n_loc, const int64_t *rowptr, const int32_t *col,
                  const double *r, const double *c, const double *v,
                  const double *X, int64_t F, double *Y)
{
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < n_loc; ++i) {
        double *y = Y + i * F;
        for (int64_t f = 0; f < F; ++f) y[f] = 0.0;
        for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
            int64_t j = col[e];
            double w = (v ? v[e] : 1.0) * c[j];
            const double *x = X + j * F;
            for (int64_t f = 0; f < F; ++f) y[f] += w * x[f];
        }
        for (int64_t f = 0; f < F; ++f) y[f] *= r[i];
    }
}

/* dX[j,f] = c[j] * sum_{e: col[e]=j, increasing e} v[e] * r[row(e)] * dY[row(e), f], for every j < n_cols.
 * Edges are visited in increasing e; threads split the feature columns, never the edges. */
void orc_spmm_bwd(int64_t n_loc, int64_t n_cols, const int64_t *rowptr, const int32_t *col,
                  const double *r, const double *c, const double *v,
                  const double *dY, int64_t F, double *dX)
{
    int nt = orc_max_threads();
    if (nt > F) nt = (int)(F > 0 ? F : 1);
#pragma omp parallel for schedule(static) num_threads(nt)
    for (int t = 0; t < nt; ++t) {
        int64_t f0 = F * t / nt, f1 = F * (t + 1) / nt;
        for (int64_t j = 0; j < n_cols; ++j)
            for (int64_t f = f0; f < f1; ++f) dX[j * F + f] = 0.0;
        for (int64_t i = 0; i < n_loc; ++i) {
            const double *g = dY + i * F;
            for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
                double w = (v ? v[e] : 1.0) * r[i];
                double *d = dX + (int64_t)col[e] * F;
                for (int64_t f = f0; f < f1; ++f) d[f] += w * g[f];
            }
        }
        for (int64_t j = 0; j < n_cols; ++j)
            for (int64_t f = f0; f < f1; ++f) dX[j * F + f] *= c[j];
    }
}

/* ---------------------------------------------------------------- loss (O7) */
/* L = (1/norm) * sum_{i masked} (logsumexp(Z_i) - Z_i[y_i]);  dZ_i = (softmax(Z_i) - e_{y_i}) / norm
 * on masked rows, 0 elsewhere.  norm <= 0 means "number of masked rows".  mask == NULL: all rows. */
double orc_softmax_ce(int64_t n, int64_t C, const double *Z, const int32_t *y, const uint8_t *mask,
                      double norm, double *dZ)
{
    if (norm <= 0.0) {
        int64_t cnt = 0;
        for (int64_t i = 0; i < n; ++i) cnt += (!mask || mask[i]) ? 1 : 0;
        norm = cnt > 0 ? (double)cnt : 1.0;
    }
    double loss = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        const double *z = Z + i * C;
        double *g = dZ ? dZ + i * C : NULL;
        if (mask && !mask[i]) {
            if (g) for (int64_t k = 0; k < C; ++k) g[k] = 0.0;
            continue;
        }
        double m = z[0];
        for (int64_t k = 1; k < C; ++k) if (z[k] > m) m = z[k];
        double s = 0.0;
        for (int64_t k = 0; k < C; ++k) s += exp(z[k] - m);
        double lse = m + log(s);
        loss += lse - z[y[i]];
        if (g) {
            for (int64_t k = 0; k < C; ++k) g[k] = exp(z[k] - lse) / norm;
            g[y[i]] -= 1.0 / norm;
        }
    }
    return loss / norm;
}
