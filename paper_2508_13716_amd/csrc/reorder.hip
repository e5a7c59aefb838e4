// Storage order of a partition's vertices (the subgraph reordering step that follows RAPA, reorder figure) and the
// CSR relabelling that goes with it.  Host code: it runs once, before the graph handle is created.
//
// The paper asks only for an order with better memory access; two are offered.
//   POPULARITY  sorts each range (local, halo) by how many entries refer to a vertex.  The feature rows that
//               the aggregation gathers most often then sit next to each other, which helps the address
//               translation caches and the DRAM page hit rate; it needs no structure in the graph.
//   BFS         numbers the local vertices in breadth-first order and the halo vertices by first use.  Vertices
//               that are neighbours in the graph get nearby places, so rows processed together gather from a
//               narrow range of the operand and find each other's lines in the L2.
#include "common.h"

#include <algorithm>
#include <numeric>
#include <vector>

using namespace capgnn;

static int check_csr(const char *who, int64_t n_loc, int64_t n_halo, const int64_t *rowptr, const int32_t *col) {
    if (n_loc < 0 || n_halo < 0 || !rowptr) CG_FAIL(CAPGNN_EINVAL, "%s: bad sizes or NULL rowptr", who);
    const int64_t n_cols = n_loc + n_halo;
    if (n_cols >= (int64_t(1) << 31) - 1) CG_FAIL(CAPGNN_EINVAL, "%s: n_loc+n_halo must be < 2^31-1", who);
    if (rowptr[0] != 0) CG_FAIL(CAPGNN_EINVAL, "%s: rowptr[0] must be 0", who);
    for (int64_t i = 0; i < n_loc; ++i)
        if (rowptr[i + 1] < rowptr[i]) CG_FAIL(CAPGNN_EINVAL, "%s: rowptr decreases at row %lld", who, (long long)i);
    const int64_t nnz = rowptr[n_loc];
    if (nnz > 0 && !col) CG_FAIL(CAPGNN_EINVAL, "%s: col is NULL", who);
    for (int64_t e = 0; e < nnz; ++e)
        if (col[e] < 0 || col[e] >= n_cols)
            CG_FAIL(CAPGNN_EINVAL, "%s: col[%lld]=%d outside [0,%lld)", who, (long long)e, col[e], (long long)n_cols);
    return CAPGNN_OK;
}

extern "C" int capgnn_locality_order(int method, int64_t n_loc, int64_t n_halo, const int64_t *rowptr,
                                     const int32_t *col, int32_t *new2old) {
    CG_TRY(check_csr("locality_order", n_loc, n_halo, rowptr, col));
    if (!new2old && n_loc + n_halo > 0) CG_FAIL(CAPGNN_EINVAL, "locality_order: new2old is NULL");
    const int64_t n_cols = n_loc + n_halo, nnz = rowptr[n_loc];
    if (method == CAPGNN_RELABEL_POPULARITY) {
        std::vector<int64_t> refs(n_cols, 0);
        for (int64_t e = 0; e < nnz; ++e) ++refs[col[e]];
        std::iota(new2old, new2old + n_cols, 0);
        auto more_refs = [&](int32_t a, int32_t b) { return refs[a] > refs[b]; };   // stable: ties keep index order
        std::stable_sort(new2old, new2old + n_loc, more_refs);
        std::stable_sort(new2old + n_loc, new2old + n_cols, more_refs);
        return CAPGNN_OK;
    }
    if (method != CAPGNN_RELABEL_BFS) CG_FAIL(CAPGNN_EINVAL, "locality_order: unknown method %d", method);
    std::vector<int32_t> roots(n_loc);
    std::iota(roots.begin(), roots.end(), 0);
    std::stable_sort(roots.begin(), roots.end(), [&](int32_t a, int32_t b) {
        return rowptr[a + 1] - rowptr[a] > rowptr[b + 1] - rowptr[b];
    });
    std::vector<uint8_t> placed(n_cols, 0);
    int64_t tail = 0, head = 0;   // the filled part of new2old is the queue of the search
    for (int32_t r : roots) {
        if (placed[r]) continue;
        placed[r] = 1;
        new2old[tail++] = r;
        for (; head < tail; ++head) {
            const int32_t u = new2old[head];
            for (int64_t e = rowptr[u]; e < rowptr[u + 1]; ++e) {
                const int32_t v = col[e];
                if (v < n_loc && !placed[v]) {
                    placed[v] = 1;
                    new2old[tail++] = v;
                }
            }
        }
    }
    for (int64_t k = 0; k < n_loc; ++k) {
        const int32_t u = new2old[k];
        for (int64_t e = rowptr[u]; e < rowptr[u + 1]; ++e) {
            const int32_t v = col[e];
            if (v >= n_loc && !placed[v]) {
                placed[v] = 1;
                new2old[tail++] = v;
            }
        }
    }
    for (int64_t v = n_loc; v < n_cols; ++v)
        if (!placed[v]) new2old[tail++] = static_cast<int32_t>(v);
    return CAPGNN_OK;
}

extern "C" int capgnn_relabel_csr(int64_t n_loc, int64_t n_halo, const int64_t *rowptr, const int32_t *col,
                                  const float *edge_val, const int32_t *new2old, int64_t *rowptr_out,
                                  int32_t *col_out, float *val_out) {
    CG_TRY(check_csr("relabel_csr", n_loc, n_halo, rowptr, col));
    const int64_t n_cols = n_loc + n_halo;
    if (!new2old && n_cols > 0) CG_FAIL(CAPGNN_EINVAL, "relabel_csr: new2old is NULL");
    if (!rowptr_out || (rowptr[n_loc] > 0 && !col_out)) CG_FAIL(CAPGNN_EINVAL, "relabel_csr: NULL output");
    if (edge_val && !val_out && rowptr[n_loc] > 0) CG_FAIL(CAPGNN_EINVAL, "relabel_csr: edge_val given but val_out is NULL");
    std::vector<int32_t> old2new(n_cols, -1);
    for (int64_t k = 0; k < n_cols; ++k) {
        const int32_t o = new2old[k];
        const bool in_range = k < n_loc ? (o >= 0 && o < n_loc) : (o >= n_loc && o < n_cols);
        if (!in_range || old2new[o] >= 0)
            CG_FAIL(CAPGNN_EINVAL, "relabel_csr: new2old[%lld]=%d is repeated or leaves its range", (long long)k, o);
        old2new[o] = static_cast<int32_t>(k);
    }
    rowptr_out[0] = 0;
    std::vector<std::pair<int32_t, int64_t>> row;   // (new column, old entry): sorting it orders equal columns by entry
    for (int64_t k = 0; k < n_loc; ++k) {
        const int64_t o = new2old[k];
        row.clear();
        for (int64_t e = rowptr[o]; e < rowptr[o + 1]; ++e) row.emplace_back(old2new[col[e]], e);
        std::sort(row.begin(), row.end());
        int64_t q = rowptr_out[k];
        for (const auto &en : row) {
            col_out[q] = en.first;
            if (edge_val) val_out[q] = edge_val[en.second];
            ++q;
        }
        rowptr_out[k + 1] = q;
    }
    return CAPGNN_OK;
}
