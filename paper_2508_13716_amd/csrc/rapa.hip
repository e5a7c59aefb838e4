// RAPA's subgraph adjustment (Alg. 2 do_partition around Alg. 3 adjust_subgraph) with the cost model of Eq. 3-5, and the
// two small graph operations around it (edges per halo vertex; the subgraph without the removed halo vertices).
// Host code: integer bookkeeping and a handful of double-precision costs per removal.  The halo vertices are ranked by
// the influence score of Eq. 6, which the caller computes with capgnn_influence_score (an SpMV-shaped kernel) and
// passes in: a removal costs O(1) here because a subgraph's cost depends only on its vertex and edge counts.
#include "common.h"

#include <algorithm>
#include <cmath>
#include <numeric>

// costs are compared with thresholds, so they are formed exactly as written: no fused multiply-adds
#pragma clang fp contract(off)

namespace capgnn {

struct RapaState {
    int64_t n_inner, e_inner;
    int64_t e_outer;     // edges of the halo vertices still in the subgraph
    int64_t n_kept;      // halo vertices still in the subgraph
};

struct RapaRatios {      // a GPU's measured costs divided by the largest among the GPUs
    double spmm, mm, h2d, d2h, idt;
};

static double rapa_lambda(const RapaState &s, const RapaRatios &q, double alpha, int P) {
    const double e_all = static_cast<double>(s.e_inner + s.e_outer);
    const double t_comm = static_cast<double>(s.e_outer) * ((q.h2d + q.d2h) * (1.0 - 1.0 / P) + q.idt * (1.0 / P));
    const double t_comp = alpha * e_all * q.spmm + (1.0 - alpha) * static_cast<double>(s.n_inner) * q.mm;
    return t_comp + t_comm;
}

static bool rapa_mem_ok(const RapaState &s, const capgnn_rapa_device &d, const capgnn_rapa_params &p) {
    const double nv = static_cast<double>(s.n_inner + s.n_kept), ne = static_cast<double>(s.e_inner + s.e_outer);
    const double need = nv * p.m_vertex + ne * p.m_edge + nv * static_cast<double>(p.f_dim) * p.m_feat + p.beta;
    return d.mem_bytes >= need;
}

}  // namespace capgnn

using namespace capgnn;

extern "C" int capgnn_halo_edge_counts(int64_t n_loc, int64_t n_halo, const int64_t *rowptr, const int32_t *col,
                                       int64_t *e_inner, int64_t *halo_edges) {
    if (n_loc < 0 || n_halo < 0 || !rowptr || !e_inner || (n_halo > 0 && !halo_edges)) CG_FAIL(CAPGNN_EINVAL, "halo_edge_counts: bad argument");
    const int64_t nnz = rowptr[n_loc];
    if (nnz > 0 && !col) CG_FAIL(CAPGNN_EINVAL, "halo_edge_counts: col is NULL");
    std::fill(halo_edges, halo_edges + n_halo, int64_t(0));
    int64_t inner = 0;
    for (int64_t e = 0; e < nnz; ++e) {
        const int64_t c = col[e];
        if (c < 0 || c >= n_loc + n_halo) CG_FAIL(CAPGNN_EINVAL, "halo_edge_counts: column %lld out of range", static_cast<long long>(c));
        if (c < n_loc) ++inner;
        else ++halo_edges[c - n_loc];
    }
    *e_inner = inner;
    return CAPGNN_OK;
}

extern "C" int capgnn_prune_halo(int64_t n_loc, int64_t n_halo, const int64_t *rowptr, const int32_t *col,
                                 const uint8_t *keep, int64_t *rowptr_out, int32_t *col_out, int64_t *new_index) {
    if (n_loc < 0 || n_halo < 0 || !rowptr || !rowptr_out || (n_halo > 0 && (!keep || !new_index)))
        CG_FAIL(CAPGNN_EINVAL, "prune_halo: bad argument");
    const int64_t nnz = rowptr[n_loc];
    if (nnz > 0 && (!col || !col_out)) CG_FAIL(CAPGNN_EINVAL, "prune_halo: col is NULL");
    int64_t q = 0;
    for (int64_t k = 0; k < n_halo; ++k) new_index[k] = keep[k] ? q++ : -1;
    int64_t w = 0;
    rowptr_out[0] = 0;
    for (int64_t i = 0; i < n_loc; ++i) {
        for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
            const int64_t c = col[e];
            if (c < 0 || c >= n_loc + n_halo) CG_FAIL(CAPGNN_EINVAL, "prune_halo: column %lld out of range", static_cast<long long>(c));
            if (c < n_loc) col_out[w++] = static_cast<int32_t>(c);
            else if (keep[c - n_loc]) col_out[w++] = static_cast<int32_t>(n_loc + new_index[c - n_loc]);
        }
        rowptr_out[i + 1] = w;
    }
    return CAPGNN_OK;
}

extern "C" int capgnn_rapa_adjust(int n_parts, const int64_t *n_inner, const int64_t *e_inner, const int64_t *halo_ptr,
                                  const int64_t *halo_edges, const float *score, const capgnn_rapa_device *dev,
                                  const capgnn_rapa_params *prm, uint8_t *keep, double *lambda_out, int32_t *r_out,
                                  int *sweeps_out, double *sigma_out) {
    if (n_parts <= 0 || !n_inner || !e_inner || !halo_ptr || !dev || !prm) CG_FAIL(CAPGNN_EINVAL, "rapa_adjust: NULL argument");
    const int P = n_parts;
    const int64_t n_h = halo_ptr[P];
    if (halo_ptr[0] != 0 || n_h < 0 || (n_h > 0 && (!halo_edges || !score || !keep))) CG_FAIL(CAPGNN_EINVAL, "rapa_adjust: bad halo arrays");
    if (!(prm->alpha >= 0.0 && prm->alpha <= 1.0) || prm->max_sweeps <= 0) CG_FAIL(CAPGNN_EINVAL, "rapa_adjust: alpha must lie in [0,1], max_sweeps > 0");
    capgnn_rapa_device mx = dev[0];
    for (int i = 0; i < P; ++i) {
        if (halo_ptr[i + 1] < halo_ptr[i] || n_inner[i] < 0 || e_inner[i] < 0) CG_FAIL(CAPGNN_EINVAL, "rapa_adjust: bad sizes of subgraph %d", i);
        const capgnn_rapa_device &d = dev[i];
        if (!(d.t_spmm > 0 && d.t_mm > 0 && d.f_h2d > 0 && d.f_d2h > 0 && d.f_idt > 0))
            CG_FAIL(CAPGNN_EINVAL, "rapa_adjust: the measured costs of GPU %d must be positive", i);
        mx.t_spmm = std::max(mx.t_spmm, d.t_spmm); mx.t_mm = std::max(mx.t_mm, d.t_mm);
        mx.f_h2d = std::max(mx.f_h2d, d.f_h2d); mx.f_d2h = std::max(mx.f_d2h, d.f_d2h); mx.f_idt = std::max(mx.f_idt, d.f_idt);
    }
    std::vector<RapaRatios> q(P);
    std::vector<RapaState> st(P);
    std::vector<std::vector<int64_t>> order(P);
    std::vector<size_t> next(P, 0);
    std::vector<double> weakness(P);
    for (int i = 0; i < P; ++i) {
        q[i] = {dev[i].t_spmm / mx.t_spmm, dev[i].t_mm / mx.t_mm, dev[i].f_h2d / mx.f_h2d, dev[i].f_d2h / mx.f_d2h,
                dev[i].f_idt / mx.f_idt};
        weakness[i] = prm->alpha * q[i].spmm + (1.0 - prm->alpha) * q[i].mm;
        const int64_t b = halo_ptr[i], n = halo_ptr[i + 1] - b;
        st[i] = {n_inner[i], e_inner[i], 0, n};
        order[i].resize(n);
        std::iota(order[i].begin(), order[i].end(), int64_t(0));
        for (int64_t k = 0; k < n; ++k) {
            if (halo_edges[b + k] < 0) CG_FAIL(CAPGNN_EINVAL, "rapa_adjust: negative edge count");
            st[i].e_outer += halo_edges[b + k];
            keep[b + k] = 1;
        }
        // ascending score, ties by index (scores compare as the floats they are passed as)
        std::stable_sort(order[i].begin(), order[i].end(), [&](int64_t a, int64_t c) { return score[b + a] < score[b + c]; });
    }
    std::vector<int> visit(P);
    std::iota(visit.begin(), visit.end(), 0);
    std::stable_sort(visit.begin(), visit.end(), [&](int a, int c) { return weakness[a] > weakness[c]; });   // weakest GPU first

    auto mean_lambda = [&]() {
        double s = 0.0;
        for (int j = 0; j < P; ++j) s += rapa_lambda(st[j], q[j], prm->alpha, P);
        return s / P;
    };
    int sweeps = 0;
    double sigma = 0.0;
    std::vector<int32_t> r(P, 0);
    for (;;) {
        std::fill(r.begin(), r.end(), 0);
        for (int i : visit) {                                        // ---- Alg. 3
            const double lam_i = rapa_lambda(st[i], q[i], prm->alpha, P);
            const double lam_bar = mean_lambda();
            if (lam_i <= lam_bar && rapa_mem_ok(st[i], dev[i], *prm)) { r[i] = 1; continue; }
            const int64_t b = halo_ptr[i];
            int64_t removed = 0;
            double lam_hat = lam_i;
            while (lam_hat > lam_bar && next[i] < order[i].size()) {
                const int64_t k = order[i][next[i]++];
                keep[b + k] = 0;
                st[i].e_outer -= halo_edges[b + k];
                st[i].n_kept -= 1;
                ++removed;
                lam_hat = rapa_lambda(st[i], q[i], prm->alpha, P);
                if (lam_hat <= 0.5 * (lam_i + lam_bar) && rapa_mem_ok(st[i], dev[i], *prm)) break;
            }
            if (removed == 0) r[i] = 1;
        }
        ++sweeps;                                                    // ---- Alg. 2
        const double mean = mean_lambda();
        double var = 0.0;
        for (int j = 0; j < P; ++j) {
            const double d = rapa_lambda(st[j], q[j], prm->alpha, P) - mean;
            var += d * d;
        }
        sigma = std::sqrt(var / P);
        const bool all_done = std::all_of(r.begin(), r.end(), [](int32_t v) { return v == 1; });
        if (sigma < prm->epsilon || all_done || sweeps >= prm->max_sweeps) break;
    }
    for (int i = 0; i < P; ++i) {
        if (lambda_out) lambda_out[i] = rapa_lambda(st[i], q[i], prm->alpha, P);
        if (r_out) r_out[i] = r[i];
    }
    if (sweeps_out) *sweeps_out = sweeps;
    if (sigma_out) *sigma_out = sigma;
    return CAPGNN_OK;
}
