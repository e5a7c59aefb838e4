// Layer forward / backward and the epoch: host-side orchestration of the kernels.
//
// A_hat X W can be associated two ways.  AGG_FIRST runs the SpMM at width f_in and the GEMM over the
// n_loc local rows, and needs no transposed SpMM when the layer's input gradient is not wanted (the
// first layer).  XFORM_FIRST runs the GEMM over all n_cols rows and the SpMM at width f_out.  Both
// give the same result in exact arithmetic; the choice is a cost decision (capgnn_layer_order).
#include "common.h"
#include <memory>

#include <algorithm>
#include <cstring>

namespace capgnn {

// Row pitch (in elements) of the library's own matrices: rows start on 16-byte boundaries; a row shorter than a
// cache line gets a whole line when that costs at most a third more memory (96-byte rows at a 96-byte pitch
// straddle two lines three times out of four; C4's 47-wide aggregation gains 8 %).  Wider rows keep the 16-byte
// pitch: padding 400-byte rows to 512 made C3's dense products 12 % slower.
// When the graph has a column-blocked copy the pitch is a whole, odd number of 128-byte lines: the blocked kernel
// gathers the same 128-byte slice of many rows at a time; the slices then coincide with cache lines (C2's 41-wide
// launch 0.57 -> 0.44 ms) and, with an odd line count, spread over all sixteen channels of an L2 instead of one or
// two (C2's 256-wide launches 1.88 -> 1.70 ms).
static int pad_ld(const capgnn_graph *g, int f, int dtype) {
    const int es = elem_bytes(dtype);
    const int bytes16 = (f * es + 15) / 16 * 16;
    int bytes = (bytes16 < 128 && (128 - bytes16) * 3 <= bytes16) ? 128 : bytes16;
    if (g->fwd.ncb || g->bwd.ncb) {
        bytes = (bytes + 127) / 128 * 128;          // slices of the blocked kernel coincide with cache lines
        if (bytes % 256 == 0) bytes += 128;
    }
    return bytes / es;
}

// Event-pair recorder for per-kernel timings (only active when the caller asks for times).
struct Recorder {
    struct Rec { int kind, layer, backward; hipEvent_t e0, e1; };
    std::vector<Rec> recs;
    std::vector<hipEvent_t> pool;
    size_t used = 0;
    bool on = false;

    hipEvent_t get() {
        if (used == pool.size()) {
            hipEvent_t e = nullptr;
            if (hipEventCreate(&e) != hipSuccess) return nullptr;
            pool.push_back(e);
        }
        return pool[used++];
    }
    void reset(bool enable) { recs.clear(); used = 0; on = enable; }
    void begin(int kind, int layer, int backward, hipStream_t st) {
        if (!on) return;
        Rec r{kind, layer, backward, get(), get()};
        if (r.e0 && r.e1) {
            (void)hipEventRecord(r.e0, st);
            recs.push_back(r);
        }
    }
    void end(hipStream_t st) {
        if (!on || recs.empty()) return;
        (void)hipEventRecord(recs.back().e1, st);
    }
};

static thread_local Recorder g_rec;

struct Scope {
    hipStream_t st;
    Scope(int kind, int layer, int backward, hipStream_t s) : st(s) { g_rec.begin(kind, layer, backward, s); }
    ~Scope() { g_rec.end(st); }
};

static int check_layer(const capgnn_graph *g, const capgnn_layer *l, const char *who) {
    if (!g || !l) CG_FAIL(CAPGNN_EINVAL, "%s: NULL graph or layer", who);
    if (l->kind != CAPGNN_GCN && l->kind != CAPGNN_SAGE_MEAN) CG_FAIL(CAPGNN_EINVAL, "%s: unknown layer kind %d", who, l->kind);
    if (l->f_in <= 0 || l->f_out <= 0) CG_FAIL(CAPGNN_EINVAL, "%s: bad layer widths", who);
    if (l->dtype != CAPGNN_F32 && l->dtype != CAPGNN_BF16) CG_FAIL(CAPGNN_EINVAL, "%s: unknown dtype", who);
    if (l->act != CAPGNN_ACT_NONE && l->act != CAPGNN_ACT_RELU) CG_FAIL(CAPGNN_EINVAL, "%s: unknown activation", who);
    if (l->order < CAPGNN_ORDER_AUTO || l->order > CAPGNN_XFORM_FIRST) CG_FAIL(CAPGNN_EINVAL, "%s: unknown order", who);
    if (!l->W) CG_FAIL(CAPGNN_EINVAL, "%s: W is NULL", who);
    if (l->kind == CAPGNN_SAGE_MEAN && !l->W_self) CG_FAIL(CAPGNN_EINVAL, "%s: W_self is NULL for a SAGE layer", who);
    return CAPGNN_OK;
}

// Cost model behind ORDER_AUTO: gathered bytes at an effective cache-served rate plus matrix-core time.
static int resolve_order(const capgnn_graph *g, const capgnn_layer *l, int need_dx) {
    if (l->order != CAPGNN_ORDER_AUTO) return l->order;
    const double s = elem_bytes(l->dtype);
    const double bw = 3.0e12, fl = 60.0e12;
    const double nnz = static_cast<double>(g->nnz), nl = static_cast<double>(g->n_loc), nc = static_cast<double>(g->n_cols);
    const double fi = l->f_in, fo = l->f_out;
    const double gemm_loc = 2.0 * nl * fi * fo / fl, gemm_all = 2.0 * nc * fi * fo / fl;
    const double agg = nnz * fi * s / bw + 2.0 * gemm_loc + (need_dx ? gemm_loc + nnz * fi * s / bw : 0.0);
    const double xf = 2.0 * gemm_all + 2.0 * nnz * fo * s / bw + (need_dx ? gemm_loc : 0.0);
    return agg <= xf ? CAPGNN_AGG_FIRST : CAPGNN_XFORM_FIRST;
}

static size_t saved_bytes(const capgnn_graph *g, const capgnn_layer *l, int order) {
    if (order == CAPGNN_XFORM_FIRST) return 0;
    return align_up(static_cast<size_t>(g->n_loc) * pad_ld(g, l->f_in, l->dtype) * elem_bytes(l->dtype), 256);
}

// forward scratch: [transformed features T (XFORM_FIRST)] [scratch of the aggregation kernel]
static size_t fwd_t_bytes(const capgnn_graph *g, const capgnn_layer *l, int order) {
    if (order == CAPGNN_AGG_FIRST) return 0;
    return align_up(static_cast<size_t>(g->n_cols) * pad_ld(g, l->f_out, l->dtype) * elem_bytes(l->dtype), 256);
}

// scratch of the transform GEMMs (the bf16 kernel lays the weight out with the reduction index contiguous)
static size_t fwd_g_bytes(const capgnn_graph *g, const capgnn_layer *l) {
    const size_t b = gemm_ws_bytes(0, g->n_cols, l->f_out, l->f_in);
    // a GraphSAGE layer's two fp32 products run as one launch over both weight matrices
    return (l->kind == CAPGNN_SAGE_MEAN && l->dtype == CAPGNN_F32) ? std::max(b, gemm_dual_ws_bytes(l->f_out, l->f_in, l->f_in)) : b;
}

static size_t fwd_ws_bytes(const capgnn_graph *g, const capgnn_layer *l, int order) {
    return fwd_t_bytes(g, l, order) + fwd_g_bytes(g, l) +
           spmm_ws_bytes(g->fwd, order == CAPGNN_AGG_FIRST ? l->f_in : l->f_out, l->dtype);
}

// A bf16 layer that stores its output as float (the layer that feeds the loss) also takes its output gradient as
// float: the loss gradient's values cluster around (p - 1) / n and p / n, so rounding them to bf16 before they are
// summed over millions of vertices shifts every term the same way (measured on the 2.45 M-vertex configuration: 2 % of
// the last weight gradient, against 0.02 % when only the aggregated gradient is rounded).  The transposed aggregation
// reads the float rows and rounds its result once; the dense products that need a bf16 operand read this copy.
static size_t grad_copy_bytes(const capgnn_graph *g, const capgnn_layer *l) {
    if (!(l->dtype == CAPGNN_BF16 && l->out_f32)) return 0;
    return align_up(static_cast<size_t>(g->n_loc) * pad_ld(g, l->f_out, CAPGNN_BF16) * sizeof(uint16_t), 256);
}

static size_t bwd_ws_bytes(const capgnn_graph *g, const capgnn_layer *l, int order) {
    const int es = elem_bytes(l->dtype);
    size_t b = relu_bias_ws_bytes(g->n_loc, l->f_out);
    const int64_t red_rows = order == CAPGNN_AGG_FIRST ? g->n_loc : g->n_cols;
    b += std::max(std::max(gemm_ws_bytes(1, l->f_in, l->f_out, red_rows), gemm_ws_bytes(1, l->f_in, l->f_out, g->n_loc)),
                  gemm_ws_bytes(0, g->n_cols, l->f_in, l->f_out));
    if (order == CAPGNN_AGG_FIRST) b += align_up(static_cast<size_t>(g->n_loc) * pad_ld(g, l->f_in, l->dtype) * es, 256);
    else b += align_up(static_cast<size_t>(g->n_cols) * pad_ld(g, l->f_out, l->dtype) * es, 256);
    b += spmm_ws_bytes(g->bwd, order == CAPGNN_AGG_FIRST ? l->f_in : l->f_out, l->dtype);
    b += grad_copy_bytes(g, l);
    return b;
}

static int layer_fwd_impl(const capgnn_graph *g, const capgnn_layer *l, int order, int li, const void *X, int64_t ldx,
                          void *H, int64_t ldh, void *saved, void *ws, size_t ws_bytes, hipStream_t st) {
    const int dt = l->dtype, es = elem_bytes(dt);
    const bool sage = l->kind == CAPGNN_SAGE_MEAN;
    const int relu = l->act == CAPGNN_ACT_RELU;
    if (!X || !H) CG_FAIL(CAPGNN_EINVAL, "layer_fwd: NULL operand");
    if (ldx < l->f_in || ldh < l->f_out) CG_FAIL(CAPGNN_EINVAL, "layer_fwd: leading dimension too small");
    if (order == CAPGNN_AGG_FIRST) {
        if (!saved) CG_FAIL(CAPGNN_EINVAL, "layer_fwd: saved is NULL (AGG_FIRST keeps the aggregated input)");
        const int64_t ldm = pad_ld(g, l->f_in, dt);
        {
            Scope s(CAPGNN_K_SPMM_FWD, li, 0, st);
            SpmmEpilogue ep;
            if (ws && ws_bytes >= fwd_ws_bytes(g, l, order)) {
                ep.ws = static_cast<char *>(ws) + fwd_g_bytes(g, l);
                ep.ws_bytes = ws_bytes - fwd_g_bytes(g, l);
            }
            CG_TRY(launch_spmm(g->fwd, false, X, ldx, saved, ldm, l->f_in, dt, ep, st));
        }
        Scope s(CAPGNN_K_GEMM, li, 0, st);
        void *gws = (ws && ws_bytes >= fwd_g_bytes(g, l)) ? ws : nullptr;
        const size_t gwb = gws ? fwd_g_bytes(g, l) : 0;
        if (sage)       // H = act(M W + X_loc W_self + b): one launch where the three-piece fp32 form applies
            return launch_gemm_dual(g->n_loc, l->f_out, l->f_in, saved, ldm, l->W, l->f_out, l->f_in, X, ldx, l->W_self, l->f_out,
                                    H, ldh, dt, l->out_f32, l->bias, relu, gws, gwb, st, l->f32_product);
        CG_TRY(launch_gemm(0, 0, g->n_loc, l->f_out, l->f_in, saved, ldm, l->W, l->f_out, H, ldh, dt, l->out_f32, 0, l->bias,
                           relu, nullptr, 0, gws, gwb, st, nullptr, l->f32_product));
        return CAPGNN_OK;
    }
    // XFORM_FIRST.  When an entry's weight depends on its source alone (no edge values), the product's epilogue
    // multiplies row s of T by that weight and the aggregation sums unweighted: its entry list is half as long to read.
    // fp32 only: a bf16 T would round the scaled rows a second time.
    const bool pre = dt == CAPGNN_F32 && g->fwd.weights_by_source;
    const int64_t ldt = pad_ld(g, l->f_out, dt);
    const size_t need = fwd_ws_bytes(g, l, order);
    if (!ws || ws_bytes < need) CG_FAIL(CAPGNN_ENOMEM, "layer_fwd: workspace of %zu bytes needed, %zu given", need, ws_bytes);
    (void)es;
    {
        Scope s(CAPGNN_K_GEMM, li, 0, st);
        void *gws = static_cast<char *>(ws) + fwd_t_bytes(g, l, order);
        CG_TRY(launch_gemm(0, 0, g->n_cols, l->f_out, l->f_in, X, ldx, l->W, l->f_out, ws, ldt, dt, 0, 0, nullptr, 0,
                           nullptr, 0, gws, fwd_g_bytes(g, l), st, pre ? g->fwd.in_scale : nullptr, l->f32_product));
        if (sage)
            CG_TRY(launch_gemm(0, 0, g->n_loc, l->f_out, l->f_in, X, ldx, l->W_self, l->f_out, H, ldh, dt, l->out_f32, 0,
                               nullptr, 0, nullptr, 0, gws, fwd_g_bytes(g, l), st, nullptr, l->f32_product));
    }
    Scope s(CAPGNN_K_SPMM_FWD, li, 0, st);
    SpmmEpilogue ep;
    ep.bias = l->bias; ep.relu = relu; ep.accumulate = sage ? 1 : 0; ep.out_f32 = l->out_f32;
    ep.operand_scaled = pre;
    ep.ws = static_cast<char *>(ws) + fwd_t_bytes(g, l, order) + fwd_g_bytes(g, l);
    ep.ws_bytes = ws_bytes - fwd_t_bytes(g, l, order) - fwd_g_bytes(g, l);
    CG_TRY(launch_spmm(g->fwd, false, ws, ldt, H, ldh, l->f_out, dt, ep, st));
    return CAPGNN_OK;
}

static int layer_bwd_impl(const capgnn_graph *g, const capgnn_layer *l, int order, int li, const void *X, int64_t ldx,
                          const void *H, int64_t ldh, const void *saved, void *dH, int64_t lddh, float *dW,
                          float *dW_self, float *dbias, void *dX, int64_t lddx, int need_halo_grad, void *ws,
                          size_t ws_bytes, hipStream_t st) {
    const int dt = l->dtype;
    const bool sage = l->kind == CAPGNN_SAGE_MEAN;
    const int relu = l->act == CAPGNN_ACT_RELU;
    if (!X || !dH || (relu && !H)) CG_FAIL(CAPGNN_EINVAL, "layer_bwd: NULL operand");
    if (ldx < l->f_in || lddh < l->f_out || (dX && lddx < l->f_in)) CG_FAIL(CAPGNN_EINVAL, "layer_bwd: leading dimension too small");
    if (ws_bytes < bwd_ws_bytes(g, l, order) || !ws)
        CG_FAIL(CAPGNN_ENOMEM, "layer_bwd: workspace of %zu bytes needed, %zu given", bwd_ws_bytes(g, l, order), ws_bytes);
    char *w = static_cast<char *>(ws);
    void *ws_rb = w;
    const size_t rb = relu_bias_ws_bytes(g->n_loc, l->f_out);
    w += rb;
    const int64_t red_rows = order == CAPGNN_AGG_FIRST ? g->n_loc : g->n_cols;
    const size_t gw = std::max(std::max(gemm_ws_bytes(1, l->f_in, l->f_out, red_rows), gemm_ws_bytes(1, l->f_in, l->f_out, g->n_loc)),
                               gemm_ws_bytes(0, g->n_cols, l->f_in, l->f_out));
    void *ws_gemm = w;
    w += gw;
    void *tmp = w;   // dM (AGG_FIRST) or dT (XFORM_FIRST)
    w += order == CAPGNN_AGG_FIRST ? align_up(static_cast<size_t>(g->n_loc) * pad_ld(g, l->f_in, dt) * elem_bytes(dt), 256)
                                   : align_up(static_cast<size_t>(g->n_cols) * pad_ld(g, l->f_out, dt) * elem_bytes(dt), 256);
    // float output gradient of a bf16 layer (see grad_copy_bytes): dZ stays float for the transposed aggregation; the
    // dense products read its rounded copy
    const bool f32grad = dt == CAPGNN_BF16 && l->out_f32;
    void *dHb = dH;                 // the gradient as the dense products read it (storage type of the layer)
    int64_t lddhb = lddh;
    if (f32grad) {
        dHb = w;
        lddhb = pad_ld(g, l->f_out, CAPGNN_BF16);
        w += grad_copy_bytes(g, l);
    }
    SpmmEpilogue sp_ep;   // scratch of the transposed aggregation
    sp_ep.ws = w;
    sp_ep.ws_bytes = ws_bytes - static_cast<size_t>(w - static_cast<char *>(ws));

    // The transposed aggregation weighs an entry by the scale of its (local) source row alone when the operator has no
    // edge values: the rows it gathers are multiplied by that scale where they are produced (dZ below when it is
    // gathered itself and nothing else reads it; dH W^T in the other order) and it sums unweighted.  fp32 only.
    const bool pre_b = dt == CAPGNN_F32 && g->bwd.weights_by_source;
    const bool scale_dz = pre_b && order == CAPGNN_XFORM_FIRST && !sage && (dW || dX);
    const bool need_copy = f32grad && (order == CAPGNN_AGG_FIRST || sage);
    {   // dZ = dH * sigma'(Z) in place; dbias = column sums of dZ
        Scope s(CAPGNN_K_ELEMENTWISE, li, 1, st);
        const int h_dt = (l->out_f32 ? CAPGNN_F32 : dt);
        if (f32grad) {
            // mask and bias gradient in float, in place; then the rounded copy where a dense product needs one
            CG_TRY(launch_relu_mask_dbias(g->n_loc, l->f_out, nullptr, 0, CAPGNN_F32, dH, lddh, H, ldh, CAPGNN_F32, h_dt, relu,
                                          dbias, ws_rb, rb, st, nullptr));
            if (need_copy)
                CG_TRY(launch_relu_mask_dbias(g->n_loc, l->f_out, dH, lddh, CAPGNN_F32, dHb, lddhb, nullptr, 0, CAPGNN_BF16,
                                              h_dt, 0, nullptr, ws_rb, rb, st, nullptr));
        } else {
            CG_TRY(launch_relu_mask_dbias(g->n_loc, l->f_out, nullptr, 0, dt, dH, lddh, H, ldh, dt, h_dt, relu, dbias,
                                          ws_rb, rb, st, scale_dz ? g->bwd.in_scale : nullptr));
        }
    }
    if (order == CAPGNN_AGG_FIRST) {
        if (!saved) CG_FAIL(CAPGNN_EINVAL, "layer_bwd: saved is NULL");
        const int64_t ldm = pad_ld(g, l->f_in, dt);
        {
            Scope s(CAPGNN_K_GEMM, li, 1, st);
            if (dW) CG_TRY(launch_gemm(1, 0, l->f_in, l->f_out, g->n_loc, saved, ldm, dHb, lddhb, dW, l->f_out, dt, 1, 0,
                                       nullptr, 0, nullptr, 0, ws_gemm, gw, st, nullptr, l->f32_product));
            if (sage && dW_self)
                CG_TRY(launch_gemm(1, 0, l->f_in, l->f_out, g->n_loc, X, ldx, dHb, lddhb, dW_self, l->f_out, dt, 1, 0,
                                   nullptr, 0, nullptr, 0, ws_gemm, gw, st, nullptr, l->f32_product));
            if (dX) CG_TRY(launch_gemm(0, 1, g->n_loc, l->f_in, l->f_out, dHb, lddhb, l->W, l->f_out, tmp, ldm, dt, 0, 0,
                                       nullptr, 0, nullptr, 0, ws_gemm, gw, st, pre_b ? g->bwd.in_scale : nullptr, l->f32_product));
        }
        if (dX) {
            {
                Scope s(CAPGNN_K_SPMM_BWD, li, 1, st);
                sp_ep.operand_scaled = pre_b;
                CG_TRY(launch_spmm(g->bwd, !need_halo_grad, tmp, ldm, dX, lddx, l->f_in, dt, sp_ep, st));
            }
            if (sage) {
                Scope s(CAPGNN_K_GEMM, li, 1, st);
                CG_TRY(launch_gemm(0, 1, g->n_loc, l->f_in, l->f_out, dHb, lddhb, l->W_self, l->f_out, dX, lddx, dt, 0, 1,
                                   nullptr, 0, nullptr, 0, ws_gemm, gw, st, nullptr, l->f32_product));
            }
        }
        return CAPGNN_OK;
    }
    // XFORM_FIRST: dT = A_hat^T dZ over all columns, then dW = X^T dT, dX = dT W^T
    const int64_t ldt = pad_ld(g, l->f_out, dt);
    if (dW || dX) {
        Scope s(CAPGNN_K_SPMM_BWD, li, 1, st);
        const bool sub = !dW && !need_halo_grad;
        sp_ep.operand_scaled = scale_dz;
        sp_ep.out_bf16 = f32grad;       // float rows in, one rounding on the way out
        CG_TRY(launch_spmm(g->bwd, sub, dH, lddh, tmp, ldt, l->f_out, f32grad ? CAPGNN_F32 : dt, sp_ep, st));
    }
    Scope s(CAPGNN_K_GEMM, li, 1, st);
    if (dW) CG_TRY(launch_gemm(1, 0, l->f_in, l->f_out, g->n_cols, X, ldx, tmp, ldt, dW, l->f_out, dt, 1, 0, nullptr, 0,
                               nullptr, 0, ws_gemm, gw, st, nullptr, l->f32_product));
    if (sage && dW_self)
        CG_TRY(launch_gemm(1, 0, l->f_in, l->f_out, g->n_loc, X, ldx, dHb, lddhb, dW_self, l->f_out, dt, 1, 0, nullptr, 0,
                           nullptr, 0, ws_gemm, gw, st, nullptr, l->f32_product));
    if (dX) {
        const int64_t rows = need_halo_grad ? g->n_cols : g->n_loc;
        CG_TRY(launch_gemm(0, 1, rows, l->f_in, l->f_out, tmp, ldt, l->W, l->f_out, dX, lddx, dt, 0, 0, nullptr, 0,
                           nullptr, 0, ws_gemm, gw, st, nullptr, l->f32_product));
        if (sage)
            CG_TRY(launch_gemm(0, 1, g->n_loc, l->f_in, l->f_out, dHb, lddhb, l->W_self, l->f_out, dX, lddx, dt, 0, 1,
                               nullptr, 0, nullptr, 0, ws_gemm, gw, st, nullptr, l->f32_product));
    }
    return CAPGNN_OK;
}

// ------------------------------------------------------------------ epoch workspace plan
struct EpochPlan {
    std::vector<int> order;
    std::vector<int64_t> ldx;          // leading dimension of layer l's input
    std::vector<size_t> x_off, saved_off;
    size_t logits_off = 0, dz32_off = 0, grad_off[2] = {0, 0}, layer_ws_off = 0, layer_ws_bytes = 0, loss_ws_off = 0,
           loss_val_off = 0, staging_off = 0, total = 0;
    int64_t ld_grad = 0, ldz = 0;
};

static int plan_epoch(const capgnn_graph *g, const capgnn_cache *c, const capgnn_layer *layers, int L, int64_t ld0,
                      EpochPlan *p) {
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes, 256); return o; };
    p->order.resize(L); p->ldx.resize(L); p->x_off.assign(L, 0); p->saved_off.assign(L, 0);
    int64_t max_w = 0;
    size_t lws = 0;
    for (int l = 0; l < L; ++l) {
        const capgnn_layer *ly = &layers[l];
        p->order[l] = resolve_order(g, ly, l > 0);
        p->ldx[l] = l == 0 ? ld0 : pad_ld(g, ly->f_in, ly->dtype);
        if (l > 0) p->x_off[l] = take(static_cast<size_t>(g->n_cols) * p->ldx[l] * elem_bytes(ly->dtype));
        p->saved_off[l] = take(saved_bytes(g, ly, p->order[l]));
        max_w = std::max<int64_t>(max_w, std::max(pad_ld(g, ly->f_out, ly->dtype), l > 0 ? pad_ld(g, ly->f_in, ly->dtype) : 0));
        lws = std::max(lws, std::max(fwd_ws_bytes(g, ly, p->order[l]), bwd_ws_bytes(g, ly, p->order[l])));
    }
    p->ldz = pad_ld(g, layers[L - 1].f_out, CAPGNN_F32);
    p->logits_off = take(static_cast<size_t>(g->n_loc) * p->ldz * sizeof(float));
    // a bf16 model keeps the loss gradient in float: the last layer's backward pass reads it unrounded
    if (layers[0].dtype == CAPGNN_BF16) p->dz32_off = take(static_cast<size_t>(g->n_loc) * p->ldz * sizeof(float));
    p->ld_grad = max_w;
    p->grad_off[0] = take(static_cast<size_t>(g->n_loc) * max_w * sizeof(float));
    p->grad_off[1] = take(static_cast<size_t>(g->n_loc) * max_w * sizeof(float));
    p->layer_ws_bytes = lws;
    p->layer_ws_off = take(lws);
    p->loss_ws_off = take(capgnn_loss_workspace_bytes(g->n_loc));
    p->loss_val_off = take(256);
    if (c && c->miss_mode != CAPGNN_MISS_ZEROCOPY) {
        size_t hb = 0;
        for (int l = 0; l < c->n_layers; ++l) hb += align_up(static_cast<size_t>(c->n_host) * c->pitch[l], 256);
        p->staging_off = take(hb);
    }
    p->total = off;
    return CAPGNN_OK;
}

static int check_epoch_args(const capgnn_graph *g, const capgnn_cache *c, const capgnn_layer *layers, int L) {
    if (!g || !layers || L <= 0 || L > 16) CG_FAIL(CAPGNN_EINVAL, "epoch: bad graph / layers / L");
    if ((g->n_halo > 0) != (c != nullptr)) CG_FAIL(CAPGNN_EINVAL, "epoch: cache must be given iff the partition has halo vertices");
    for (int l = 0; l < L; ++l) {
        CG_TRY(check_layer(g, &layers[l], "epoch"));
        if (layers[l].dtype != layers[0].dtype) CG_FAIL(CAPGNN_EINVAL, "epoch: all layers must share one dtype");
        if (l > 0 && layers[l].f_in != layers[l - 1].f_out) CG_FAIL(CAPGNN_EINVAL, "epoch: layer %d input width != layer %d output width", l, l - 1);
        if (l < L - 1 && layers[l].out_f32) CG_FAIL(CAPGNN_EINVAL, "epoch: out_f32 is only meaningful on the last layer");
    }
    if (c) {
        if (c->n_halo != g->n_halo) CG_FAIL(CAPGNN_EINVAL, "epoch: cache and graph disagree on n_halo");
        if (c->n_layers < L) CG_FAIL(CAPGNN_EINVAL, "epoch: cache holds %d layer tables, model has %d layers", c->n_layers, L);
        if (c->dtype != layers[0].dtype) CG_FAIL(CAPGNN_EINVAL, "epoch: cache dtype differs from the layers' dtype");
        for (int l = 0; l < L; ++l)
            if (c->dims[l] != layers[l].f_in) CG_FAIL(CAPGNN_EINVAL, "epoch: cache table %d has width %d, layer input has %d", l, c->dims[l], layers[l].f_in);
    }
    return CAPGNN_OK;
}

}  // namespace capgnn

using namespace capgnn;

extern "C" int capgnn_layer_order(const capgnn_graph *g, const capgnn_layer *l, int need_dx) {
    if (check_layer(g, l, "layer_order") != CAPGNN_OK) return CAPGNN_EINVAL;
    return resolve_order(g, l, need_dx);
}

extern "C" size_t capgnn_layer_saved_bytes(const capgnn_graph *g, const capgnn_layer *l) {
    if (!g || !l) return 0;
    // the order may be resolved with or without an input gradient: reserve for the larger case
    return std::max(saved_bytes(g, l, resolve_order(g, l, 0)), saved_bytes(g, l, resolve_order(g, l, 1)));
}

extern "C" size_t capgnn_layer_workspace_bytes(const capgnn_graph *g, const capgnn_layer *l) {
    if (!g || !l) return 0;
    size_t b = 0;
    for (int o : {CAPGNN_AGG_FIRST, CAPGNN_XFORM_FIRST}) {
        if (l->order != CAPGNN_ORDER_AUTO && l->order != o) continue;
        b = std::max(b, std::max(fwd_ws_bytes(g, l, o), bwd_ws_bytes(g, l, o)));
    }
    return b;
}

extern "C" int capgnn_layer_fwd(const capgnn_graph *g, const capgnn_layer *l, const void *X, int64_t ldx, void *H,
                                int64_t ldh, void *saved, void *ws, size_t ws_bytes, void *stream) {
    CG_TRY(check_layer(g, l, "layer_fwd"));
    if (l->order == CAPGNN_ORDER_AUTO) CG_FAIL(CAPGNN_EINVAL, "layer_fwd: resolve ORDER_AUTO with capgnn_layer_order() first, forward and backward must agree");
    g_rec.reset(false);
    return layer_fwd_impl(g, l, l->order, 0, X, ldx, H, ldh, saved, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

extern "C" int capgnn_layer_bwd(const capgnn_graph *g, const capgnn_layer *l, const void *X, int64_t ldx, const void *H,
                                int64_t ldh, const void *saved, void *dH, int64_t lddh, float *dW, float *dW_self,
                                float *dbias, void *dX, int64_t lddx, int need_halo_grad, void *ws, size_t ws_bytes,
                                void *stream) {
    CG_TRY(check_layer(g, l, "layer_bwd"));
    if (l->order == CAPGNN_ORDER_AUTO) CG_FAIL(CAPGNN_EINVAL, "layer_bwd: resolve ORDER_AUTO with capgnn_layer_order() first, forward and backward must agree");
    g_rec.reset(false);
    return layer_bwd_impl(g, l, l->order, 0, X, ldx, H, ldh, saved, dH, lddh, dW, dW_self, dbias, dX, lddx,
                          need_halo_grad, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

extern "C" size_t capgnn_epoch_workspace_bytes(const capgnn_graph *g, const capgnn_cache *c, const capgnn_layer *layers,
                                               int L) {
    if (check_epoch_args(g, c, layers, L) != CAPGNN_OK) return 0;
    EpochPlan p;
    // ld0 does not enter the plan's sizes (layer 0 reads the caller's buffer)
    plan_epoch(g, c, layers, L, layers[0].f_in, &p);
    return p.total;
}

extern "C" int capgnn_epoch_activation(const capgnn_graph *g, const capgnn_cache *c, const capgnn_layer *layers, int L,
                                       int l, void *ws, void **ptr, int64_t *ld) {
    CG_TRY(check_epoch_args(g, c, layers, L));
    if (l < 0 || l >= L - 1 || !ws || !ptr || !ld) CG_FAIL(CAPGNN_EINVAL, "epoch_activation: bad argument (hidden layers are 0..L-2)");
    EpochPlan p;
    plan_epoch(g, c, layers, L, layers[0].f_in, &p);
    *ptr = static_cast<char *>(ws) + p.x_off[l + 1];
    *ld = p.ldx[l + 1];
    return CAPGNN_OK;
}

// labels (class indices, softmax cross-entropy) or targets (0/1 matrix, binary cross-entropy): exactly one is given
// The events that order the two streams of an epoch.  An eager epoch uses the cache's own; an epoch that is being
// recorded into a HIP graph brings a set of its own (an event last recorded during a capture must not be waited for
// outside it) and sets `capture`.
struct EpochEvents {
    hipEvent_t fork = nullptr, join = nullptr;
    std::vector<hipEvent_t> layer, consumed;
    bool capture = false;
};

static int epoch_impl(const capgnn_graph *g, capgnn_cache *c, const capgnn_layer *layers, int L, void *X0,
                      int64_t ld0, const int32_t *labels, const uint8_t *targets, int64_t ldt, const uint8_t *mask,
                      double loss_norm, float *logits, float **dW, float **dW_self, float **dbias, float lr, float *loss_out,
                      capgnn_epoch_times *times, void *ws, size_t ws_bytes, void *stream, void *side_stream,
                      const EpochEvents *own_events = nullptr) {
    CG_TRY(check_epoch_args(g, c, layers, L));
    if (!X0 || (!labels && !targets) || !dW || !dbias) CG_FAIL(CAPGNN_EINVAL, "epoch: NULL argument");
    if (targets && ldt < layers[L - 1].f_out) CG_FAIL(CAPGNN_EINVAL, "epoch: ldt smaller than the number of classes");
    if (ld0 < layers[0].f_in) CG_FAIL(CAPGNN_EINVAL, "epoch: ld0 smaller than the input width");
    const int dt = layers[0].dtype, es = elem_bytes(dt);
    if (dt == CAPGNN_BF16 && !layers[L - 1].out_f32) CG_FAIL(CAPGNN_EINVAL, "epoch: the last bf16 layer must set out_f32 (the loss reads float logits)");
    if (lr != 0.f && dt != CAPGNN_F32) CG_FAIL(CAPGNN_EUNSUPPORTED, "epoch: the in-place SGD step needs float weights");
    EpochPlan p;
    plan_epoch(g, c, layers, L, ld0, &p);
    if (!ws || ws_bytes < p.total) CG_FAIL(CAPGNN_ENOMEM, "epoch: workspace of %zu bytes needed, %zu given", p.total, ws_bytes);
    if (reinterpret_cast<uintptr_t>(ws) & 255u) CG_FAIL(CAPGNN_EINVAL, "epoch: workspace must be 256-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipStream_t side = side_stream ? static_cast<hipStream_t>(side_stream) : st;
    char *w = static_cast<char *>(ws);
    const int C = layers[L - 1].f_out;
    float *Z = reinterpret_cast<float *>(w + p.logits_off);   // padded pitch keeps the vector paths usable
    const int64_t ldz = p.ldz;
    void *staging = (c && c->miss_mode != CAPGNN_MISS_ZEROCOPY) ? w + p.staging_off : nullptr;
    g_rec.reset(times != nullptr);
    hipEvent_t ev_t0 = nullptr, ev_t1 = nullptr;
    if (times) {
        ev_t0 = g_rec.get(); ev_t1 = g_rec.get();
        if (!ev_t0 || !ev_t1) CG_FAIL(CAPGNN_EHIP, "epoch: hipEventCreate failed");
        CG_HIP(hipEventRecord(ev_t0, st));
    }
    auto Xl = [&](int l) -> char * { return l == 0 ? static_cast<char *>(X0) : w + p.x_off[l]; };

    // host-tier rows of every layer start moving now, on the side stream, ahead of the layers that use them
    const bool has_miss = c && c->n_host > 0;
    // pipelined: the rows were copied into the staging area while the previous epoch ran; each area is
    // refilled for the next epoch as soon as this epoch has scattered it
    const bool pipelined = has_miss && c->miss_mode == CAPGNN_MISS_PIPELINED && side != st;
    auto halo_rows = [&](int l) -> char * { return Xl(l) + static_cast<size_t>(g->n_loc) * p.ldx[l] * es; };
    EpochEvents cache_events;
    if (!own_events && c) {
        cache_events.fork = c->ev_fork; cache_events.join = c->ev_join;
        cache_events.layer = c->ev_layer; cache_events.consumed = c->ev_consumed;
    }
    const EpochEvents &ev = own_events ? *own_events : cache_events;
    const bool capture = ev.capture;
    if (has_miss && side != st) {
        if (pipelined && capture) {
            // a recorded epoch consumes what the run before it prefetched: that must exist when the first replay starts
            bool primed = c->staged_base == staging;
            for (int l = 0; l < L; ++l) primed = primed && c->staged_valid[l];
            if (!primed)
                CG_FAIL(CAPGNN_EINVAL, "epoch: a pipelined epoch can only be recorded after one capgnn_epoch with the same ws and "
                                       "side stream has prefetched the host tier");
        }
        CG_HIP(hipEventRecord(ev.fork, st));
        CG_HIP(hipStreamWaitEvent(side, ev.fork, 0));
        if (!capture) c->last_side = side;
        if (pipelined) {
            if (c->staged_base != staging) {
                std::fill(c->staged_valid.begin(), c->staged_valid.end(), 0);
                c->staged_base = staging;
            }
            for (int l = 0; l < L; ++l) {
                if (c->staged_valid[l]) continue;
                Scope s(CAPGNN_K_GATHER_MISS, l, 0, side);     // cold start: nothing was prefetched for this layer
                CG_TRY(stage_misses(c, l, staging, side));
                CG_HIP(hipEventRecord(ev.layer[l], side));
                c->staged_valid[l] = 1;
            }
        } else {
            for (int l = 0; l < L; ++l) {
                Scope s(CAPGNN_K_GATHER_MISS, l, 0, side);
                CG_TRY(gather_all_misses(c, l, halo_rows(l), p.ldx[l], staging, side));
                if (!g_rec.on) CG_HIP(hipEventRecord(ev.layer[l], side));
            }
        }
    }
    // forward
    for (int l = 0; l < L; ++l) {
        char *X = Xl(l);
        char *halo = halo_rows(l);
        if (c) {
            if (pipelined) {
                // the staged rows landed while the previous epoch ran: both device-resident sources in one launch.  (In a
                // recorded epoch the replay before this one ended only after its prefetches had: nothing to wait for.)
                if (!capture) CG_HIP(hipStreamWaitEvent(st, ev.layer[l], 0));
                {
                    Scope s(CAPGNN_K_GATHER_HIT, l, 0, st);
                    CG_TRY(gather_hits_and_staged(c, l, halo, p.ldx[l], staging, st));
                }
                CG_HIP(hipEventRecord(ev.consumed[l], st));
                CG_HIP(hipStreamWaitEvent(side, ev.consumed[l], 0));
                Scope s(CAPGNN_K_GATHER_MISS, l, 0, side);     // the next epoch's rows of this layer
                CG_TRY(stage_misses(c, l, staging, side));
                CG_HIP(hipEventRecord(ev.layer[l], side));
            } else {
                Scope s(CAPGNN_K_GATHER_HIT, l, 0, st);
                CG_TRY(gather_all_hits(c, l, halo, p.ldx[l], st));
            }
            if (!pipelined && has_miss) {
                if (side != st) {
                    if (g_rec.on) {
                        // the recorder's stop event of this layer's transfer doubles as the join point
                        for (auto &r : g_rec.recs)
                            if (r.kind == CAPGNN_K_GATHER_MISS && r.layer == l) CG_HIP(hipStreamWaitEvent(st, r.e1, 0));
                    } else {
                        CG_HIP(hipStreamWaitEvent(st, ev.layer[l], 0));
                    }
                } else {
                    Scope s(CAPGNN_K_GATHER_MISS, l, 0, st);
                    CG_TRY(gather_all_misses(c, l, halo, p.ldx[l], staging, st));
                }
            }
        }
        const bool last = l == L - 1;
        void *Hout = last ? static_cast<void *>(Z) : static_cast<void *>(Xl(l + 1));
        const int64_t ldh = last ? ldz : p.ldx[l + 1];
        CG_TRY(layer_fwd_impl(g, &layers[l], p.order[l], l, X, p.ldx[l], Hout, ldh, w + p.saved_off[l],
                              w + p.layer_ws_off, p.layer_ws_bytes, st));
    }
    // loss and its gradient w.r.t. the logits
    float *loss_dev = reinterpret_cast<float *>(w + p.loss_val_off);
    int cur = 0;
    {
        Scope s(CAPGNN_K_LOSS, L - 1, 0, st);
        // a bf16 model gets the gradient in fp32 first (the bias gradient is summed before rounding)
        void *dz = dt == CAPGNN_BF16 ? static_cast<void *>(w + p.dz32_off) : static_cast<void *>(w + p.grad_off[cur]);
        const int64_t lddz = dt == CAPGNN_BF16 ? ldz : p.ld_grad;
        const int dzt = dt == CAPGNN_BF16 ? CAPGNN_F32 : dt;
        if (targets)
            CG_TRY(capgnn_sigmoid_bce(g->n_loc, C, Z, ldz, targets, ldt, mask, loss_norm, loss_dev, dz, lddz, dzt,
                                      w + p.loss_ws_off, capgnn_loss_workspace_bytes(g->n_loc), st));
        else    // the loss kernel reads every logit anyway: it also writes the caller's dense copy
            CG_TRY(softmax_ce_with_copy(g->n_loc, C, Z, ldz, labels, mask, loss_norm, loss_dev, dz, lddz, dzt,
                                        w + p.loss_ws_off, capgnn_loss_workspace_bytes(g->n_loc), st, logits));
    }
    // backward
    for (int l = L - 1; l >= 0; --l) {
        const bool last = l == L - 1;
        const void *Hl = last ? static_cast<const void *>(Z) : static_cast<const void *>(Xl(l + 1));
        const int64_t ldh = last ? ldz : p.ldx[l + 1];
        void *dX = l > 0 ? static_cast<void *>(w + p.grad_off[cur ^ 1]) : nullptr;
        // the last layer of a bf16 model takes the loss gradient as float (its output is float as well)
        const bool f32grad = last && dt == CAPGNN_BF16;
        CG_TRY(layer_bwd_impl(g, &layers[l], p.order[l], l, Xl(l), p.ldx[l], Hl, ldh, w + p.saved_off[l],
                              f32grad ? static_cast<void *>(w + p.dz32_off) : static_cast<void *>(w + p.grad_off[cur]),
                              f32grad ? ldz : p.ld_grad, dW[l], dW_self ? dW_self[l] : nullptr, dbias[l], dX,
                              p.ld_grad, 0, w + p.layer_ws_off, p.layer_ws_bytes, st));
        cur ^= 1;
    }
    if (lr != 0.f) {
        Scope s(CAPGNN_K_ELEMENTWISE, 0, 1, st);
        for (int l = 0; l < L; ++l) {
            const int64_t nw = static_cast<int64_t>(layers[l].f_in) * layers[l].f_out;
            CG_TRY(launch_sgd(static_cast<float *>(layers[l].W), dW[l], nw, lr, st));
            if (layers[l].kind == CAPGNN_SAGE_MEAN && dW_self && dW_self[l])
                CG_TRY(launch_sgd(static_cast<float *>(layers[l].W_self), dW_self[l], nw, lr, st));
            if (layers[l].bias && dbias[l]) CG_TRY(launch_sgd(layers[l].bias, dbias[l], layers[l].f_out, lr, st));
        }
    }
    if (logits && targets)
        CG_HIP(hipMemcpy2DAsync(logits, static_cast<size_t>(C) * sizeof(float), Z, static_cast<size_t>(ldz) * sizeof(float),
                                static_cast<size_t>(C) * sizeof(float), static_cast<size_t>(g->n_loc),
                                hipMemcpyDeviceToDevice, st));
    if (capture && has_miss && side != st) {
        // a recorded epoch ends when its side stream has: the prefetches for the next replay are part of this one
        CG_HIP(hipEventRecord(ev.join, side));
        CG_HIP(hipStreamWaitEvent(st, ev.join, 0));
    }
    if (times) CG_HIP(hipEventRecord(ev_t1, st));
    if (loss_out) {
        CG_HIP(hipMemcpyAsync(loss_out, loss_dev, sizeof(float), hipMemcpyDeviceToHost, st));
        CG_HIP(hipStreamSynchronize(st));
    }
    if (times) {
        CG_HIP(hipStreamSynchronize(st));
        if (side != st) CG_HIP(hipStreamSynchronize(side));
        std::memset(times, 0, sizeof(*times));
        CG_HIP(hipEventElapsedTime(&times->total_ms, ev_t0, ev_t1));
        for (const auto &r : g_rec.recs) {
            float ms = 0.f;
            CG_HIP(hipEventElapsedTime(&ms, r.e0, r.e1));
            switch (r.kind) {
                case CAPGNN_K_GATHER_HIT: case CAPGNN_K_GATHER_STAGED: times->pick_cache_ms += ms; break;
                case CAPGNN_K_GATHER_MISS: times->communication_ms += ms; break;
                case CAPGNN_K_SPMM_FWD: case CAPGNN_K_SPMM_BWD: times->aggregation_ms += ms; break;
                case CAPGNN_K_GEMM: times->combine_ms += ms; break;
                case CAPGNN_K_LOSS: times->loss_ms += ms; break;
                default: times->other_ms += ms; break;
            }
            if (times->n_records < CAPGNN_MAX_RECORDS) {
                auto &o = times->records[times->n_records++];
                o.kind = r.kind; o.layer = r.layer; o.backward = r.backward; o.ms = ms;
            }
        }
        g_rec.reset(false);
    }
    return CAPGNN_OK;
}

extern "C" int capgnn_epoch(const capgnn_graph *g, capgnn_cache *c, const capgnn_layer *layers, int L, void *X0,
                            int64_t ld0, const int32_t *labels, const uint8_t *mask, double loss_norm, float *logits,
                            float **dW, float **dW_self, float **dbias, float lr, float *loss_out,
                            capgnn_epoch_times *times, void *ws, size_t ws_bytes, void *stream, void *side_stream) {
    if (!labels) CG_FAIL(CAPGNN_EINVAL, "epoch: labels is NULL");
    return epoch_impl(g, c, layers, L, X0, ld0, labels, nullptr, 0, mask, loss_norm, logits, dW, dW_self, dbias, lr, loss_out,
                      times, ws, ws_bytes, stream, side_stream);
}

extern "C" int capgnn_epoch_multilabel(const capgnn_graph *g, capgnn_cache *c, const capgnn_layer *layers, int L, void *X0,
                                       int64_t ld0, const uint8_t *targets, int64_t ldt, const uint8_t *mask,
                                       double loss_norm, float *logits, float **dW, float **dW_self, float **dbias,
                                       float lr, float *loss_out, capgnn_epoch_times *times, void *ws, size_t ws_bytes,
                                       void *stream, void *side_stream) {
    if (!targets) CG_FAIL(CAPGNN_EINVAL, "epoch_multilabel: targets is NULL");
    return epoch_impl(g, c, layers, L, X0, ld0, nullptr, targets, ldt, mask, loss_norm, logits, dW, dW_self, dbias, lr,
                      loss_out, times, ws, ws_bytes, stream, side_stream);
}

// ---- the epoch as a HIP graph: one launch per epoch instead of one per kernel

struct capgnn_epoch_graph {
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
    EpochEvents ev;                 // the events the recorded epoch orders its two streams with
    capgnn_cache *cache = nullptr;  // whose eager epochs may have left work on their side stream
    hipEvent_t side_done = nullptr;

    ~capgnn_epoch_graph() {
        if (side_done) (void)hipEventDestroy(side_done);
        if (exec) (void)hipGraphExecDestroy(exec);
        if (graph) (void)hipGraphDestroy(graph);
        if (ev.fork) (void)hipEventDestroy(ev.fork);
        if (ev.join) (void)hipEventDestroy(ev.join);
        for (hipEvent_t e : ev.layer) if (e) (void)hipEventDestroy(e);
        for (hipEvent_t e : ev.consumed) if (e) (void)hipEventDestroy(e);
    }
};

__global__ void copy_loss_kernel(const float *src, float *dst) { *dst = *src; }

extern "C" int capgnn_epoch_graph_create(capgnn_epoch_graph **out, const capgnn_graph *g, capgnn_cache *c,
                                         const capgnn_layer *layers, int L, void *X0, int64_t ld0, const int32_t *labels,
                                         const uint8_t *mask, double loss_norm, float *logits, float **dW, float **dW_self,
                                         float **dbias, float lr, float *loss_dev, void *ws, size_t ws_bytes, void *stream,
                                         void *side_stream) {
    if (!out) CG_FAIL(CAPGNN_EINVAL, "epoch_graph_create: out is NULL");
    *out = nullptr;
    if (!stream) CG_FAIL(CAPGNN_EINVAL, "epoch_graph_create: a stream of the caller's is needed (the default stream cannot be captured)");
    if (!labels) CG_FAIL(CAPGNN_EINVAL, "epoch_graph_create: labels is NULL");
    CG_TRY(check_epoch_args(g, c, layers, L));
    hipStream_t st = static_cast<hipStream_t>(stream);
    std::unique_ptr<capgnn_epoch_graph> eg(new capgnn_epoch_graph);
    eg->ev.capture = true;
    eg->ev.layer.assign(L, nullptr);
    eg->ev.consumed.assign(L, nullptr);
    bool ok = hipEventCreateWithFlags(&eg->ev.fork, hipEventDisableTiming) == hipSuccess &&
              hipEventCreateWithFlags(&eg->ev.join, hipEventDisableTiming) == hipSuccess;
    for (int l = 0; l < L && ok; ++l)
        ok = hipEventCreateWithFlags(&eg->ev.layer[l], hipEventDisableTiming) == hipSuccess &&
             hipEventCreateWithFlags(&eg->ev.consumed[l], hipEventDisableTiming) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&eg->side_done, hipEventDisableTiming) == hipSuccess;
    if (!ok) CG_FAIL(CAPGNN_EHIP, "epoch_graph_create: hipEventCreate failed");
    eg->cache = c;
    CG_HIP(hipStreamBeginCapture(st, hipStreamCaptureModeThreadLocal));
    // the side stream joins the recording when it waits for the epoch's first event and is joined back at the end
    int rc = epoch_impl(g, c, layers, L, X0, ld0, labels, nullptr, 0, mask, loss_norm, logits, dW, dW_self, dbias, lr, nullptr,
                        nullptr, ws, ws_bytes, stream, side_stream, &eg->ev);
    if (rc == CAPGNN_OK && loss_dev) {
        EpochPlan p;
        plan_epoch(g, c, layers, L, ld0, &p);
        hipLaunchKernelGGL(copy_loss_kernel, dim3(1), dim3(1), 0, st,
                           reinterpret_cast<const float *>(static_cast<char *>(ws) + p.loss_val_off), loss_dev);
    }
    const hipError_t e_end = hipStreamEndCapture(st, &eg->graph);       // always: the stream must leave capture mode
    if (rc != CAPGNN_OK) return rc;
    if (e_end != hipSuccess || !eg->graph) CG_FAIL(CAPGNN_EHIP, "epoch_graph_create: hipStreamEndCapture: %s", hipGetErrorString(e_end));
    const hipError_t e_inst = hipGraphInstantiate(&eg->exec, eg->graph, nullptr, nullptr, 0);
    if (e_inst != hipSuccess) CG_FAIL(CAPGNN_EHIP, "epoch_graph_create: hipGraphInstantiate: %s", hipGetErrorString(e_inst));
    *out = eg.release();
    return CAPGNN_OK;
}

extern "C" int capgnn_epoch_graph_launch(capgnn_epoch_graph *eg, void *stream) {
    if (!eg || !eg->exec) CG_FAIL(CAPGNN_EINVAL, "epoch_graph_launch: no graph");
    hipStream_t st = static_cast<hipStream_t>(stream);
    // an eager epoch before this replay may still be prefetching on its side stream into the staging area the replay reads
    if (eg->cache && eg->cache->last_side && eg->cache->last_side != st) {
        CG_HIP(hipEventRecord(eg->side_done, eg->cache->last_side));
        CG_HIP(hipStreamWaitEvent(st, eg->side_done, 0));
    }
    CG_HIP(hipGraphLaunch(eg->exec, st));
    return CAPGNN_OK;
}

extern "C" int capgnn_epoch_graph_destroy(capgnn_epoch_graph *eg) {
    delete eg;
    return CAPGNN_OK;
}
