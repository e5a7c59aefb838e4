// Cache policy layer: the vertex overlap ratio (Eq. 2) on the GPU and the two-level policy comparison
// (JACA by overlap ratio against FIFO and LRU on the same local + global structure) on the host.
#include "common.h"

#include <algorithm>
#include <numeric>

namespace capgnn {

__global__ __launch_bounds__(256) void overlap_count_kernel(const int64_t *ids, int64_t n, int64_t n_vertices, int32_t *R) {
    for (int64_t k = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; k < n; k += static_cast<int64_t>(gridDim.x) * 256) {
        const int64_t v = ids[k];
        if (v >= 0 && v < n_vertices) atomicAdd(&R[v], 1);      // integer counts: the result does not depend on the order
    }
}

__global__ __launch_bounds__(256) void fill_i32_kernel(int32_t *p, int64_t n, int32_t v) {
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; i < n; i += static_cast<int64_t>(gridDim.x) * 256)
        p[i] = v;
}

// Vertex influence score (Eq. 6): one wave per column vertex v (heaviest first).  The lanes stride over the
// entries of column v (outgoing neighbours: 1/sqrt(Din_row)) and, for a local vertex, over the entries of its
// row (incoming neighbours: 1/sqrt(Dout_col)); lane sums are combined by a butterfly in a fixed order.
struct InfluenceArgs {
    const int64_t *colptr; const int32_t *rowidx;     // CSC: entries of column v
    const int64_t *rowptr; const int32_t *col;        // CSR: entries of row i
    const int32_t *order;                              // column vertices, heaviest first
    int64_t n_loc, n_cols;
    const float *rs_din;                               // [n_loc]  1/sqrt(in-degree)
    const float *rs_dout;                              // [n_cols] 1/sqrt(out-degree)
    const float *count;                                // [n_cols] or null
    float *S;
};

__global__ __launch_bounds__(256) void influence_kernel(InfluenceArgs a) {
    const int lane = threadIdx.x & 63;
    const int64_t p = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    if (p >= a.n_cols) return;
    const int64_t v = a.order[p];
    float out_sum = 0.f, in_sum = 0.f;
    for (int64_t e = a.colptr[v] + lane; e < a.colptr[v + 1]; e += 64) out_sum += a.rs_din[a.rowidx[e]];
    if (v < a.n_loc)
        for (int64_t e = a.rowptr[v] + lane; e < a.rowptr[v + 1]; e += 64) in_sum += a.rs_dout[a.col[e]];
    for (int off = 32; off > 0; off >>= 1) {
        out_sum += __shfl_xor(out_sum, off);
        in_sum += __shfl_xor(in_sum, off);
    }
    if (lane == 0) {
        float s = out_sum * a.rs_dout[v];
        if (v < a.n_loc) s += in_sum * a.rs_din[v];
        a.S[v] = a.count ? s * a.count[v] : s;
    }
}

// A cache over the dense ids 0..n-1 with FIFO or LRU replacement: an intrusive doubly linked list from the
// next victim (head) to the newest entry (tail).
struct ListCache {
    int64_t cap = 0, size = 0;
    int32_t head = -1, tail = -1;
    std::vector<int32_t> prev, next;
    std::vector<uint8_t> in;

    void init(int64_t n, int64_t capacity) {
        cap = capacity; size = 0; head = tail = -1;
        prev.assign(n, -1); next.assign(n, -1); in.assign(n, 0);
    }
    bool has(int32_t v) const { return in[v] != 0; }
    void unlink(int32_t v) {
        if (prev[v] >= 0) next[prev[v]] = next[v]; else head = next[v];
        if (next[v] >= 0) prev[next[v]] = prev[v]; else tail = prev[v];
    }
    void push_back(int32_t v) {
        prev[v] = tail; next[v] = -1;
        if (tail >= 0) next[tail] = v; else head = v;
        tail = v;
    }
    void touch(int32_t v) { unlink(v); push_back(v); }      // LRU: a hit makes the entry the newest
    void insert(int32_t v) {
        if (cap <= 0 || in[v]) return;
        if (size >= cap) {
            const int32_t victim = head;
            unlink(victim);
            in[victim] = 0;
            --size;
        }
        push_back(v);
        in[v] = 1;
        ++size;
    }
};

}  // namespace capgnn

using namespace capgnn;

extern "C" int capgnn_overlap_ratio(const int64_t *halo_ids, int64_t n_ids, int64_t n_vertices, int32_t *R, void *stream) {
    if (n_ids < 0 || n_vertices < 0 || (n_ids > 0 && !halo_ids) || (n_vertices > 0 && !R))
        CG_FAIL(CAPGNN_EINVAL, "overlap_ratio: bad argument");
    if (n_vertices == 0) return CAPGNN_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(fill_i32_kernel, dim3(static_cast<unsigned>(std::min<int64_t>((n_vertices + 255) / 256, 4096))), dim3(256), 0, st,
                       R, n_vertices, 0);
    if (n_ids > 0)
        hipLaunchKernelGGL(overlap_count_kernel, dim3(static_cast<unsigned>(std::min<int64_t>((n_ids + 255) / 256, 8192))), dim3(256), 0,
                           st, halo_ids, n_ids, n_vertices, R);
    CG_HIP(hipGetLastError());
    return CAPGNN_OK;
}

extern "C" int capgnn_influence_score(const capgnn_graph *g, const float *inv_sqrt_din, const float *inv_sqrt_dout,
                                      const float *count, float *S, void *stream) {
    if (!g || !inv_sqrt_din || !inv_sqrt_dout || !S) CG_FAIL(CAPGNN_EINVAL, "influence_score: NULL argument");
    if (g->n_cols == 0) return CAPGNN_OK;
    InfluenceArgs a;
    a.colptr = g->bwd.ptr; a.rowidx = g->bwd.idx; a.rowptr = g->fwd.ptr; a.col = g->fwd.idx; a.order = g->bwd.order;
    a.n_loc = g->n_loc; a.n_cols = g->n_cols; a.rs_din = inv_sqrt_din; a.rs_dout = inv_sqrt_dout; a.count = count; a.S = S;
    hipLaunchKernelGGL(influence_kernel, dim3(static_cast<unsigned>((g->n_cols + 3) / 4)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), a);
    CG_HIP(hipGetLastError());
    return CAPGNN_OK;
}

extern "C" int capgnn_policy_simulate(int n_parts, const int64_t *halo_ptr, const int64_t *halo_ids, int policy,
                                      int64_t cap_local, int64_t cap_global, int epochs, int warmup, int64_t *counts) {
    if (n_parts <= 0 || !halo_ptr || !counts || epochs < 0 || warmup < 0 || policy < CAPGNN_POLICY_JACA || policy > CAPGNN_POLICY_LRU)
        CG_FAIL(CAPGNN_EINVAL, "policy_simulate: bad argument");
    if (halo_ptr[0] != 0) CG_FAIL(CAPGNN_EINVAL, "policy_simulate: halo_ptr[0] must be 0");
    const int64_t total = halo_ptr[n_parts];
    if (total > 0 && !halo_ids) CG_FAIL(CAPGNN_EINVAL, "policy_simulate: halo_ids is NULL");
    if (total >= (int64_t(1) << 31) - 1) CG_FAIL(CAPGNN_EINVAL, "policy_simulate: more than 2^31 requests per epoch");
    for (int i = 0; i < n_parts; ++i) {
        if (halo_ptr[i + 1] < halo_ptr[i]) CG_FAIL(CAPGNN_EINVAL, "policy_simulate: halo_ptr decreases");
        for (int64_t k = halo_ptr[i] + 1; k < halo_ptr[i + 1]; ++k)
            if (halo_ids[k] <= halo_ids[k - 1]) CG_FAIL(CAPGNN_EINVAL, "policy_simulate: halo set %d is not ascending and duplicate-free", i);
    }
    cap_local = std::max<int64_t>(cap_local, 0);
    cap_global = std::max<int64_t>(cap_global, 0);
    // dense ids of the union, ascending in vertex id
    std::vector<int64_t> uni(halo_ids, halo_ids + total);
    std::sort(uni.begin(), uni.end());
    uni.erase(std::unique(uni.begin(), uni.end()), uni.end());
    const int64_t U = static_cast<int64_t>(uni.size());
    std::vector<int32_t> dense(total);
    for (int64_t k = 0; k < total; ++k)
        dense[k] = static_cast<int32_t>(std::lower_bound(uni.begin(), uni.end(), halo_ids[k]) - uni.begin());
    int64_t hl = 0, hg = 0, ms = 0;
    const int counted_epochs = std::max(0, epochs - warmup);

    if (policy == CAPGNN_POLICY_JACA || policy == CAPGNN_POLICY_JACA_LOW) {
        // overlap ratio (Eq. 2), then static contents: highest (lowest) ratio first, ties by ascending vertex id
        std::vector<int32_t> R(U, 0);
        for (int64_t k = 0; k < total; ++k) ++R[dense[k]];
        const bool high = policy == CAPGNN_POLICY_JACA;
        auto before = [&](int32_t a, int32_t b) {
            if (R[a] != R[b]) return high ? R[a] > R[b] : R[a] < R[b];
            return a < b;                                          // dense ids ascend with the vertex ids
        };
        std::vector<int32_t> ord(U);
        std::iota(ord.begin(), ord.end(), 0);
        std::sort(ord.begin(), ord.end(), before);
        std::vector<uint8_t> in_glob(U, 0);
        for (int64_t k = 0; k < std::min(cap_global, U); ++k) in_glob[ord[k]] = 1;
        for (int i = 0; i < n_parts; ++i) {
            std::vector<int32_t> mine(dense.begin() + halo_ptr[i], dense.begin() + halo_ptr[i + 1]);
            std::vector<int32_t> pick(mine);
            std::sort(pick.begin(), pick.end(), before);
            std::vector<uint8_t> in_loc(U, 0);
            for (int64_t k = 0; k < std::min<int64_t>(cap_local, pick.size()); ++k) in_loc[pick[k]] = 1;
            for (int32_t v : mine) {
                if (in_loc[v]) ++hl;
                else if (in_glob[v]) ++hg;
                else ++ms;
            }
        }
        counts[0] = hl * counted_epochs; counts[1] = hg * counted_epochs; counts[2] = ms * counted_epochs;
        return CAPGNN_OK;
    }

    const bool lru = policy == CAPGNN_POLICY_LRU;
    ListCache glob;
    glob.init(U, cap_global);
    // the local cache of partition i only ever holds vertices of H_i: index it by position inside H_i
    std::vector<ListCache> loc(n_parts);
    for (int i = 0; i < n_parts; ++i) loc[i].init(halo_ptr[i + 1] - halo_ptr[i], cap_local);
    for (int e = 0; e < epochs; ++e) {
        const bool counted = e >= warmup;
        for (int i = 0; i < n_parts; ++i) {
            ListCache &lc = loc[i];
            for (int64_t k = halo_ptr[i]; k < halo_ptr[i + 1]; ++k) {
                const int32_t pos = static_cast<int32_t>(k - halo_ptr[i]), v = dense[k];
                if (lc.has(pos)) {
                    if (lru) lc.touch(pos);
                    hl += counted;
                } else if (glob.has(v)) {
                    if (lru) glob.touch(v);
                    lc.insert(pos);
                    hg += counted;
                } else {
                    glob.insert(v);
                    lc.insert(pos);
                    ms += counted;
                }
            }
        }
    }
    counts[0] = hl; counts[1] = hg; counts[2] = ms;
    return CAPGNN_OK;
}
