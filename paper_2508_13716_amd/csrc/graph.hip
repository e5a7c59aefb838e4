// Graph handle: validation, CSC construction, degree-ordered work lists, upload.
#include "common.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <numeric>

namespace capgnn {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

template <typename T>
static int upload(capgnn_graph *g, const T *host, size_t n, const T **dev_out) {
    void *d = nullptr;
    size_t bytes = std::max<size_t>(n, 1) * sizeof(T);
    if (hipMalloc(&d, bytes) != hipSuccess) CG_FAIL(CAPGNN_ENOMEM, "hipMalloc of %zu bytes failed", bytes);
    g->dev_allocs.push_back(d);
    if (n) CG_HIP(hipMemcpy(d, host, n * sizeof(T), hipMemcpyHostToDevice));
    *dev_out = static_cast<const T *>(d);
    return CAPGNN_OK;
}

// Sorting key of a row in the work lists: its entry count when that is at least EXACT_ROW, else the power of two
// below it.  Long rows are thus in exact descending order (the class limits of the kernels cut that part), and
// the many short rows of one power-of-two class stay in index order, so whatever locality the caller's vertex
// numbering has survives into the order in which rows are processed.
static int64_t order_key(int64_t len) {
    if (len >= EXACT_ROW || len <= 0) return len;
    int64_t k = 1;
    while (2 * k <= len) k *= 2;
    return k;
}

// Output rows [lo, hi) ordered by order_key (descending, ties by index); returns how many are "long".
static int64_t degree_order(const std::vector<int64_t> &ptr, int64_t lo, int64_t hi, std::vector<int32_t> &order) {
    order.resize(hi - lo);
    std::iota(order.begin(), order.end(), static_cast<int32_t>(lo));
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
        return order_key(ptr[a + 1] - ptr[a]) > order_key(ptr[b + 1] - ptr[b]);
    });
    int64_t n_long = 0;
    while (n_long < static_cast<int64_t>(order.size()) &&
           ptr[order[n_long] + 1] - ptr[order[n_long]] >= LONG_ROW)
        ++n_long;
    return n_long;
}

// Per-entry weights val * in_scale[source] (the float product the kernels would otherwise form per entry).
// Leaves *dev null when every weight is 1.
static int upload_weights(capgnn_graph *g, int64_t nnz, const int32_t *idx, const float *val, const float *in_scale,
                          const float **dev) {
    *dev = nullptr;
    if (nnz == 0 || (!val && !in_scale)) return CAPGNN_OK;
    std::vector<float> w(nnz);
    bool all_one = true;
    for (int64_t e = 0; e < nnz; ++e) {
        float x = in_scale ? in_scale[idx[e]] : 1.f;
        if (val) x *= val[e];
        w[e] = x;
        all_one = all_one && x == 1.f;
    }
    if (all_one) return CAPGNN_OK;
    return upload(g, w.data(), w.size(), dev);
}

// Cuts the leading rows of a degree-ordered work list that have at least GIANT_ROW entries into pieces.
static int upload_giant(capgnn_graph *g, const int64_t *ptr, const std::vector<int32_t> &order, GiantList *out) {
    std::vector<int32_t> pos, first(1, 0);
    int64_t n = 0;
    for (; n < static_cast<int64_t>(order.size()); ++n) {
        const int64_t len = ptr[order[n] + 1] - ptr[order[n]];
        if (len < GIANT_ROW) break;
        const int64_t pieces = (len + GIANT_PIECE - 1) / GIANT_PIECE;
        pos.insert(pos.end(), pieces, static_cast<int32_t>(n));
        first.push_back(static_cast<int32_t>(pos.size()));
    }
    if (n == 0) return CAPGNN_OK;
    CG_TRY(upload(g, pos.data(), pos.size(), &out->piece_pos));
    CG_TRY(upload(g, first.data(), first.size(), &out->piece_first));
    out->n_rows = n;
    out->n_pieces = static_cast<int64_t>(pos.size());
    return CAPGNN_OK;
}

// Column-blocked copy of one direction of the operator (see SpOp).  Worth building only when the gathered
// operand spans several blocks and a (block, row) group holds enough entries to amortise its overhead.
struct BlockedHost {
    int ncb = 0;
    int64_t n_long = 0, n_mid = 0;
    std::vector<uint32_t> off;
    std::vector<int2> ew;
    std::vector<uint16_t> src;        // ew[].x % CB_ROWS alone, for operators without edge values
};

static int32_t float_bits(float f) {
    int32_t b;
    std::memcpy(&b, &f, sizeof(b));
    return b;
}

static bool build_blocked(const int64_t *ptr, const int32_t *idx, const float *val, const float *in_scale,
                          const std::vector<int32_t> &order, int64_t n_out, int64_t n_in, BlockedHost *out) {
    const int64_t ncb = (n_in + CB_ROWS - 1) / CB_ROWS;
    const int64_t nnz = ptr[n_out];
    if (ncb < 2 || n_out == 0 || nnz / (n_out * ncb) < 16 || n_out * ncb >= (int64_t(1) << 28)) return false;
    const size_t groups = static_cast<size_t>(ncb) * n_out;
    out->ncb = static_cast<int>(ncb);
    out->off.assign(groups + 1, 0u);
    for (int64_t p = 0; p < n_out; ++p) {
        const int64_t r = order[p];
        for (int64_t e = ptr[r]; e < ptr[r + 1]; ++e) ++out->off[static_cast<size_t>(idx[e] / CB_ROWS) * n_out + p + 1];
    }
    for (size_t t = 0; t < groups; ++t) out->off[t + 1] += out->off[t];
    out->ew.resize(nnz);
    while (out->n_long < n_out && ptr[order[out->n_long] + 1] - ptr[order[out->n_long]] >= B_LONG_GROUP * ncb) ++out->n_long;
    out->n_mid = out->n_long;
    while (out->n_mid < n_out && ptr[order[out->n_mid] + 1] - ptr[order[out->n_mid]] >= B_MID_GROUP * ncb) ++out->n_mid;
    std::vector<uint32_t> cur(out->off.begin(), out->off.end() - 1);
    for (int64_t p = 0; p < n_out; ++p) {
        const int64_t r = order[p];
        for (int64_t e = ptr[r]; e < ptr[r + 1]; ++e) {
            const uint32_t q = cur[static_cast<size_t>(idx[e] / CB_ROWS) * n_out + p]++;
            float wt = in_scale ? in_scale[idx[e]] : 1.f;     // same fp32 product the unblocked kernel forms
            if (val) wt *= val[e];
            out->ew[q] = make_int2(idx[e], float_bits(wt));
        }
    }
    // Inside a group the most referenced sources come first (ties: lower index).  Most rows hold the block's
    // popular sources, so the lane groups of a wave, and the waves of a compute unit, ask for the same lines at
    // about the same time: more requests end in the L1 instead of the L2, which is what bounds the kernel.
    std::vector<int32_t> refs(n_in, 0);
    for (int64_t e = 0; e < nnz; ++e) ++refs[idx[e]];
    for (size_t t = 0; t < groups; ++t)
        std::sort(out->ew.begin() + out->off[t], out->ew.begin() + out->off[t + 1], [&](const int2 &x, const int2 &y) {
            return refs[x.x] != refs[y.x] ? refs[x.x] > refs[y.x] : x.x < y.x;
        });
    if (!val) {
        out->src.resize(nnz);
        static_assert(CB_ROWS <= 65536, "block-local row numbers are stored in 16 bits");
        for (int64_t q = 0; q < nnz; ++q) out->src[q] = static_cast<uint16_t>(out->ew[q].x % CB_ROWS);
    }
    return true;
}

static int upload_blocked(capgnn_graph *g, const BlockedHost &bh, SpOp *op) {
    CG_TRY(upload(g, bh.off.data(), bh.off.size(), &op->b_off));
    CG_TRY(upload(g, bh.ew.data(), bh.ew.size(), &op->b_ew));
    if (!bh.src.empty()) CG_TRY(upload(g, bh.src.data(), bh.src.size(), &op->b_src));
    op->ncb = bh.ncb;
    op->b_long = bh.n_long;
    op->b_mid = bh.n_mid;
    return CAPGNN_OK;
}

}  // namespace capgnn

using namespace capgnn;

extern "C" const char *capgnn_last_error(void) { return capgnn::g_err; }
extern "C" int capgnn_version(void) { return 100; }

extern "C" int capgnn_norm_scales(int kind, int64_t n_loc, int64_t n_halo, const int64_t *rowptr,
                                  const int64_t *halo_degree, float *row_scale, float *col_scale) {
    if (n_loc < 0 || n_halo < 0 || !rowptr || !row_scale || !col_scale) CG_FAIL(CAPGNN_EINVAL, "norm_scales: bad argument");
    if (kind == CAPGNN_NORM_SYM) {
        for (int64_t i = 0; i < n_loc; ++i) {
            int64_t d = std::max<int64_t>(rowptr[i + 1] - rowptr[i], 1);
            row_scale[i] = static_cast<float>(1.0 / std::sqrt(static_cast<double>(d)));
            col_scale[i] = row_scale[i];
        }
        for (int64_t h = 0; h < n_halo; ++h) {
            int64_t d = halo_degree ? std::max<int64_t>(halo_degree[h], 1) : 1;
            col_scale[n_loc + h] = static_cast<float>(1.0 / std::sqrt(static_cast<double>(d)));
        }
    } else if (kind == CAPGNN_NORM_MEAN) {
        for (int64_t i = 0; i < n_loc; ++i) {
            int64_t d = rowptr[i + 1] - rowptr[i];
            row_scale[i] = d > 0 ? static_cast<float>(1.0 / static_cast<double>(d)) : 0.0f;
        }
        for (int64_t j = 0; j < n_loc + n_halo; ++j) col_scale[j] = 1.0f;
    } else {
        CG_FAIL(CAPGNN_EINVAL, "norm_scales: unknown kind %d", kind);
    }
    return CAPGNN_OK;
}

extern "C" int capgnn_gin_operator(int64_t n_loc, int64_t n_halo, const int64_t *rowptr, const int32_t *col, float eps,
                                   int64_t *rowptr_out, int32_t *col_out, float *val_out) {
    if (n_loc < 0 || n_halo < 0 || !rowptr || !rowptr_out) CG_FAIL(CAPGNN_EINVAL, "gin_operator: bad argument");
    if (n_loc > 0 && (!col_out || !val_out)) CG_FAIL(CAPGNN_EINVAL, "gin_operator: NULL output");
    if (rowptr[0] != 0 || (rowptr[n_loc] > 0 && !col)) CG_FAIL(CAPGNN_EINVAL, "gin_operator: malformed CSR");
    rowptr_out[0] = 0;
    for (int64_t i = 0; i < n_loc; ++i) {
        if (rowptr[i + 1] < rowptr[i]) CG_FAIL(CAPGNN_EINVAL, "gin_operator: rowptr decreases at row %lld", (long long)i);
        int64_t q = rowptr_out[i];
        for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e, ++q) {
            col_out[q] = col[e];
            val_out[q] = 1.f;
        }
        col_out[q] = static_cast<int32_t>(i);
        val_out[q] = 1.f + eps;
        rowptr_out[i + 1] = q + 1;
    }
    return CAPGNN_OK;
}

extern "C" int capgnn_graph_create(capgnn_graph **out, int64_t n_loc, int64_t n_halo, const int64_t *rowptr,
                                   const int32_t *col, const float *row_scale, const float *col_scale,
                                   const float *edge_val, uint32_t flags, void *stream) {
    if (!out) CG_FAIL(CAPGNN_EINVAL, "graph_create: g is NULL");
    *out = nullptr;
    if (n_loc < 0 || n_halo < 0 || !rowptr) CG_FAIL(CAPGNN_EINVAL, "graph_create: bad sizes or NULL rowptr");
    const int64_t n_cols = n_loc + n_halo;
    if (n_cols >= (int64_t(1) << 31) - 1) CG_FAIL(CAPGNN_EINVAL, "graph_create: n_loc+n_halo must be < 2^31-1");
    if (rowptr[0] != 0) CG_FAIL(CAPGNN_EINVAL, "graph_create: rowptr[0] must be 0");
    for (int64_t i = 0; i < n_loc; ++i)
        if (rowptr[i + 1] < rowptr[i]) CG_FAIL(CAPGNN_EINVAL, "graph_create: rowptr decreases at row %lld", (long long)i);
    const int64_t nnz = rowptr[n_loc];
    if (nnz >= (int64_t(1) << 31) - 1) CG_FAIL(CAPGNN_EINVAL, "graph_create: nnz must be < 2^31-1");
    if (nnz > 0 && !col) CG_FAIL(CAPGNN_EINVAL, "graph_create: col is NULL");
    for (int64_t e = 0; e < nnz; ++e)
        if (col[e] < 0 || col[e] >= n_cols)
            CG_FAIL(CAPGNN_EINVAL, "graph_create: col[%lld]=%d outside [0,%lld)", (long long)e, col[e], (long long)n_cols);
    if ((flags & CAPGNN_GRAPH_SYMMETRIC) && n_halo != 0)
        CG_FAIL(CAPGNN_EINVAL, "graph_create: SYMMETRIC needs n_halo == 0");

    // CSC = CSR of the transpose; entries of one column keep increasing edge order
    std::vector<int64_t> colptr(n_cols + 1, 0);
    for (int64_t e = 0; e < nnz; ++e) ++colptr[col[e] + 1];
    for (int64_t j = 0; j < n_cols; ++j) colptr[j + 1] += colptr[j];
    std::vector<int32_t> rowidx(std::max<int64_t>(nnz, 1));
    std::vector<float> cscval(edge_val ? std::max<int64_t>(nnz, 1) : 0);
    {
        std::vector<int64_t> cur(colptr.begin(), colptr.end() - 1);
        for (int64_t i = 0; i < n_loc; ++i)
            for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
                int64_t p = cur[col[e]]++;
                rowidx[p] = static_cast<int32_t>(i);
                if (edge_val) cscval[p] = edge_val[e];
            }
    }
    bool share = false;
    if (flags & CAPGNN_GRAPH_SYMMETRIC) {
        bool same = std::equal(colptr.begin(), colptr.end(), rowptr) &&
                    (nnz == 0 || std::memcmp(rowidx.data(), col, nnz * sizeof(int32_t)) == 0) &&
                    (!edge_val || std::memcmp(cscval.data(), edge_val, nnz * sizeof(float)) == 0);
        if (!same) CG_FAIL(CAPGNN_EINVAL, "graph_create: SYMMETRIC flag set but the CSR differs from its transpose");
        share = true;
    }

    capgnn_graph *g = new (std::nothrow) capgnn_graph();
    if (!g) CG_FAIL(CAPGNN_ENOMEM, "graph_create: out of host memory");
    g->n_loc = n_loc; g->n_halo = n_halo; g->n_cols = n_cols; g->nnz = nnz; g->flags = flags;
    auto fail = [&](int rc) { capgnn_graph_destroy(g); return rc; };

    std::vector<int64_t> rp(rowptr, rowptr + n_loc + 1);
    std::vector<int32_t> order_f, order_b, order_bs;
    int64_t nl_f = degree_order(rp, 0, n_loc, order_f);
    int rc;
    SpOp &f = g->fwd;
    f.n_out = n_loc; f.n_in = n_cols; f.nnz = nnz; f.n_long = nl_f; f.n_sub = n_loc; f.n_long_sub = nl_f;
    if ((rc = upload(g, rowptr, n_loc + 1, &f.ptr))) return fail(rc);
    if ((rc = upload(g, col, nnz, &f.idx))) return fail(rc);
    if ((rc = upload_weights(g, nnz, col, edge_val, col_scale, &f.wt))) return fail(rc);
    f.weights_by_source = !edge_val && col_scale;
    if (row_scale && (rc = upload(g, row_scale, n_loc, &f.out_scale))) return fail(rc);
    if (col_scale && (rc = upload(g, col_scale, n_cols, &f.in_scale))) return fail(rc);
    if ((rc = upload(g, order_f.data(), order_f.size(), &f.order))) return fail(rc);
    f.order_sub = f.order;
    if ((rc = upload_giant(g, rowptr, order_f, &f.giant))) return fail(rc);
    f.giant_sub = f.giant;
    for (int64_t i = 0; i < n_loc; ++i) f.max_deg = std::max(f.max_deg, rowptr[i + 1] - rowptr[i]);
    BlockedHost bh_f;
    if (build_blocked(rowptr, col, edge_val, col_scale, order_f, n_loc, n_cols, &bh_f) && (rc = upload_blocked(g, bh_f, &f)))
        return fail(rc);

    SpOp &b = g->bwd;
    b.n_out = n_cols; b.n_in = n_loc; b.nnz = nnz; b.out_scale = f.in_scale; b.in_scale = f.out_scale;
    b.weights_by_source = !edge_val && row_scale;
    if (share) {
        b.ptr = f.ptr; b.idx = f.idx; b.order = f.order; b.n_long = f.n_long;
        b.order_sub = f.order; b.n_sub = n_loc; b.n_long_sub = f.n_long; b.max_deg = f.max_deg;
        b.giant = f.giant; b.giant_sub = f.giant;
        b.ncb = f.ncb; b.b_off = f.b_off; b.b_ew = f.b_ew; b.b_src = f.b_src; b.b_long = f.b_long; b.b_mid = f.b_mid;
        const bool same_scales = (!row_scale && !col_scale) ||
                                 (row_scale && col_scale && std::memcmp(row_scale, col_scale, n_loc * sizeof(float)) == 0);
        b.wt = f.wt;
        if (!same_scales && (rc = upload_weights(g, nnz, col, edge_val, row_scale, &b.wt))) return fail(rc);
        if (f.ncb && !same_scales) {   // the transposed product weighs an entry by the other side's scale
            if (edge_val) {
                b.ncb = 0;             // rare combination: the transposed product takes the unblocked kernel
            } else {
                for (int64_t q = 0; q < nnz; ++q) bh_f.ew[q].y = float_bits(row_scale ? row_scale[bh_f.ew[q].x] : 1.f);
                if ((rc = upload(g, bh_f.ew.data(), bh_f.ew.size(), &b.b_ew))) return fail(rc);
            }
        }
    } else {
        b.n_long = degree_order(colptr, 0, n_cols, order_b);
        b.n_long_sub = degree_order(colptr, 0, n_loc, order_bs);
        b.n_sub = n_loc;
        if ((rc = upload(g, colptr.data(), n_cols + 1, &b.ptr))) return fail(rc);
        if ((rc = upload(g, rowidx.data(), nnz, &b.idx))) return fail(rc);
        if ((rc = upload_weights(g, nnz, rowidx.data(), edge_val ? cscval.data() : nullptr, row_scale, &b.wt))) return fail(rc);
        if ((rc = upload(g, order_b.data(), order_b.size(), &b.order))) return fail(rc);
        if ((rc = upload(g, order_bs.data(), order_bs.size(), &b.order_sub))) return fail(rc);
        if ((rc = upload_giant(g, colptr.data(), order_b, &b.giant))) return fail(rc);
        if ((rc = upload_giant(g, colptr.data(), order_bs, &b.giant_sub))) return fail(rc);
        for (int64_t j = 0; j < n_cols; ++j) b.max_deg = std::max(b.max_deg, colptr[j + 1] - colptr[j]);
        BlockedHost bh;
        if (build_blocked(colptr.data(), rowidx.data(), edge_val ? cscval.data() : nullptr, row_scale, order_b, n_cols,
                          n_loc, &bh) && (rc = upload_blocked(g, bh, &b)))
            return fail(rc);
    }
    if (hipStreamSynchronize(static_cast<hipStream_t>(stream)) != hipSuccess) {
        set_error("graph_create: stream synchronisation failed");
        return fail(CAPGNN_EHIP);
    }
    *out = g;
    return CAPGNN_OK;
}

extern "C" int capgnn_graph_destroy(capgnn_graph *g) {
    if (!g) return CAPGNN_OK;
    for (void *p : g->dev_allocs) (void)hipFree(p);
    delete g;
    return CAPGNN_OK;
}
