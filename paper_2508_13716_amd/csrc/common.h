// Internal declarations shared by the translation units of libcapgnn (HIP, gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdarg.h>
#include <vector>

#include "../../include/capgnn.h"

namespace capgnn {

void set_error(const char *fmt, ...);

#define CG_FAIL(code, ...)                       \
    do {                                         \
        ::capgnn::set_error(__VA_ARGS__);        \
        return (code);                           \
    } while (0)

#define CG_HIP(expr)                                                                     \
    do {                                                                                 \
        hipError_t e__ = (expr);                                                         \
        if (e__ != hipSuccess) {                                                         \
            ::capgnn::set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e__),  \
                                __FILE__, __LINE__);                                     \
            return CAPGNN_EHIP;                                                          \
        }                                                                                \
    } while (0)

#define CG_TRY(expr)                 \
    do {                             \
        int rc__ = (expr);           \
        if (rc__ != CAPGNN_OK) return rc__; \
    } while (0)

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
static inline int elem_bytes(int dtype) { return dtype == CAPGNN_BF16 ? 2 : 4; }
static inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// One direction of the sparse operator: output row k sums over entries [ptr[k], ptr[k+1]).
// Rows of a work list that are too long for one workgroup: the first n_rows positions of the list.  Each is cut
// into pieces of GIANT_PIECE entries (the last one shorter); piece q belongs to position piece_pos[q], and the
// pieces of position p are [piece_first[p], piece_first[p+1]).
struct GiantList {
    int64_t n_rows = 0;
    int64_t n_pieces = 0;
    const int32_t *piece_pos = nullptr;    // device [n_pieces]
    const int32_t *piece_first = nullptr;  // device [n_rows + 1]
};

struct SpOp {
    int64_t n_out = 0;          // rows of the output
    int64_t n_in = 0;           // rows of the gathered operand
    int64_t nnz = 0;
    const int64_t *ptr = nullptr;     // device [n_out+1]
    const int32_t *idx = nullptr;     // device [nnz]   source row of each entry
    // device [nnz]: weight of each entry, edge value * in_scale[source] formed once (a sequential read in the
    // kernels instead of a gather from in_scale per entry); null when every weight is 1
    const float *wt = nullptr;
    // no edge values: the weight of an entry is in_scale[source] alone, so a caller that multiplies row s of the
    // operand by in_scale[s] first may ask for the unweighted sum (SpmmEpilogue::operand_scaled)
    bool weights_by_source = false;
    const float *out_scale = nullptr; // device [n_out] or null
    const float *in_scale = nullptr;  // device [n_in]  or null
    // work lists: output rows by entry count, descending; rows shorter than EXACT_ROW only by power-of-two class,
    // in index order inside a class
    const int32_t *order = nullptr;   // device [n_out]
    int64_t n_long = 0;               // first n_long entries of `order` have >= LONG_ROW entries
    int64_t n_sub = 0;                // rows [0, n_sub) of the output restricted list (bwd: local columns only)
    const int32_t *order_sub = nullptr;
    int64_t n_long_sub = 0;
    int64_t max_deg = 0;
    GiantList giant, giant_sub;       // of `order` and of `order_sub`
    // Column-blocked copy of the entries (built for dense-degree operators whose gathered operand does not
    // fit an L2): entries regrouped by (source block cb = idx / CB_ROWS, position p in `order`), original
    // entry order kept inside a group.  Group (cb, p) = entries [b_off[cb*n_out+p], b_off[cb*n_out+p+1]).
    int ncb = 0;                      // 0: no blocked copy
    const uint32_t *b_off = nullptr;  // device [ncb*n_out + 1]
    const int2 *b_ew = nullptr;       // device [nnz]  {source row, bits of the float weight val * in_scale[source]}
    // the same entries without their weights, as 16-bit row numbers inside the block (operators without edge values): read instead of b_ew when
    // every weight is 1, or when the caller has multiplied the operand rows by in_scale beforehand
    const uint16_t *b_src = nullptr;  // device [nnz] or null: source row - cb * CB_ROWS (2 bytes per entry)
    // positions [0, b_long) hold rows whose groups are long enough for a whole workgroup, [b_long, b_mid) for
    // one wave per group, the rest are walked eight rows per wave (`order` is descending in entry count)
    int64_t b_long = 0, b_mid = 0;
};

constexpr int EXACT_ROW = 256;  // work lists sort rows at least this long by their exact entry count
constexpr int LONG_ROW = 2048;  // rows at least this long are reduced by a whole workgroup
constexpr int GIANT_ROW = 16384;  // rows at least this long are cut into pieces when the caller brings scratch
constexpr int GIANT_PIECE = 4096; // entries per piece: one workgroup each, partial sums combined in piece order
constexpr int CB_ROWS = 32768;  // source rows per column block: 32768 x 128-byte slices = 4 MB, one XCD's L2 (swept: 8192 .. 49152)
constexpr int B_LONG_GROUP = 1024; // rows with at least this many entries per source block on average: workgroup per group (swept 256 .. 4096)
constexpr int B_MID_GROUP = 256;  // ... at least this many: wave per group (swept 64 .. 1024; the eight-rows-per-wave class below is the fastest)
constexpr int SLICE_BYTES = 128;  // feature bytes of one source row that one task of the blocked kernel gathers
constexpr int NUM_XCD = 8;        // L2 domains of the chip; workgroup b is dispatched to domain b % NUM_XCD

}  // namespace capgnn

struct capgnn_graph {
    int64_t n_loc = 0, n_halo = 0, n_cols = 0, nnz = 0;
    uint32_t flags = 0;
    capgnn::SpOp fwd, bwd;
    std::vector<void *> dev_allocs;
};

struct capgnn_cache {
    int64_t n_halo = 0, cap_gpu = 0, n_host = 0;
    int n_layers = 0, dtype = 0, map_kind = 0;
    std::vector<int32_t> dims;
    std::vector<int64_t> pitch;         // row pitch in bytes per layer
    std::vector<size_t> gpu_off, host_off;  // byte offset of each layer's table inside the tiers
    char *gpu_tier = nullptr;
    char *host_tier = nullptr;
    // host copies
    std::vector<int32_t> slot_h;        // [n_halo]  >=0: GPU slot, <0: host slot = -1-value
    std::vector<int64_t> gid_h;
    std::vector<int64_t> hkeys_h;       // hash table keys (gid) ...
    std::vector<int32_t> hvals_h;       // ... and halo-local index, -1 = empty
    uint64_t hmask = 0;
    // device copies
    int32_t *slot_d = nullptr;
    int32_t *gpu_list_d = nullptr;      // [cap_gpu]  halo-local index of GPU slot k
    int32_t *host_list_d = nullptr;     // [n_host]
    int64_t *hkeys_d = nullptr;
    int32_t *hvals_d = nullptr;
    int64_t *counters_d = nullptr;      // [4] hits, misses, absent
    int64_t *stamp_d = nullptr;         // [n_layers][n_halo] iteration in which each cached row was last written
    long long *owner_d = nullptr;       // [n_halo] scratch of an update call: position of the last update of a vertex
    int64_t *scan_d = nullptr;          // [n_halo/1024 + 2] scratch of the stale-list compaction
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    std::vector<hipEvent_t> ev_layer;   // one per layer: host-tier rows of that layer have landed
    std::vector<hipEvent_t> ev_consumed;  // one per layer: the layer's staging area has been scattered (pipelined mode)
    std::vector<uint8_t> staged_valid;  // pipelined mode: staging area of layer l holds rows copied for the next epoch
    void *staged_base = nullptr;        // ... inside this staging area
    hipStream_t last_side = nullptr;    // stream that may still carry such a copy
    int miss_mode = CAPGNN_MISS_STAGED;
    std::vector<void *> dev_allocs;
};

namespace capgnn {

// ---- kernels' host-side launchers (each validates what its kernel assumes) ----
struct SpmmEpilogue {
    const float *bias = nullptr;   // [F] added after scaling
    int relu = 0;
    int accumulate = 0;            // add the previous contents of Y
    int out_f32 = 0;               // store Y as float although X is bf16
    int out_bf16 = 0;              // store Y as bf16 although X is float (the loss gradient of a bf16 model is gathered unrounded)
    int operand_scaled = 0;        // row s of X already carries in_scale[s] (only for operators with weights_by_source)
    void *ws = nullptr;            // scratch for the column-blocked kernel or for cut rows (spmm_ws_bytes), may be null
    size_t ws_bytes = 0;
};

size_t spmm_ws_bytes(const SpOp &op, int F, int dtype);

int launch_spmm(const SpOp &op, bool restrict_sub, const void *X, int64_t ldx, void *Y, int64_t ldy, int F,
                int dtype, const SpmmEpilogue &ep, hipStream_t stream);

int launch_gemm(int trans_a, int trans_b, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda,
                const void *B, int64_t ldb, void *C, int64_t ldc, int dtype, int out_f32, int accumulate,
                const float *bias, int relu, const void *relu_mask, int64_t ldm, void *ws, size_t ws_bytes,
                hipStream_t stream, const float *row_scale = nullptr,    // row_scale: C[i,:] *= row_scale[i] at the very end (fp32 C)
                int f32_product = CAPGNN_F32_PRODUCT_AUTO);
// C = A W + A2 W2 (+ bias, ReLU), one launch where the fp32 three-piece form applies, else the two launches it replaces
int launch_gemm_dual(int64_t M, int64_t N, int64_t K1, const void *A, int64_t lda, const void *W, int64_t ldw, int64_t K2,
                     const void *A2, int64_t lda2, const void *W2, int64_t ldw2, void *C, int64_t ldc, int dtype, int out_f32,
                     const float *bias, int relu, void *ws, size_t ws_bytes, hipStream_t stream, int f32_product);
// scratch that lets launch_gemm_dual run as one launch
size_t gemm_dual_ws_bytes(int64_t N, int64_t K1, int64_t K2);
size_t gemm_ws_bytes(int trans_a, int64_t M, int64_t N, int64_t K);

// dZ = dH * 1[H > 0] in place (when relu) and dbias[f] = sum_i dZ[i,f] (when dbias), fixed summation order.
// src (of src_dtype, pitch lds), when non-null and different from dH, is the unrounded gradient: dH is then
// written as its masked, converted copy and the bias gradient is summed from the unrounded values.
size_t relu_bias_ws_bytes(int64_t n, int F);
int launch_relu_mask_dbias(int64_t n, int F, const void *src, int64_t lds, int src_dtype, void *dH, int64_t lddh,
                           const void *H, int64_t ldh, int dtype, int h_dtype, int relu, float *dbias, void *ws,
                           size_t ws_bytes, hipStream_t stream, const float *row_scale = nullptr);
int launch_sgd(float *W, const float *dW, int64_t n, float lr, hipStream_t stream);
// capgnn_softmax_ce that also writes the logits as a dense [n x C] matrix to `copy` (NULL: does not)
int softmax_ce_with_copy(int64_t n, int C, const float *Z, int64_t ldz, const int32_t *labels, const uint8_t *mask,
                         double loss_norm, float *loss_dev, void *dZ, int64_t lddz, int dz_dtype, void *ws, size_t ws_bytes,
                         hipStream_t st, float *copy);

uint64_t hash_gid(uint64_t x);

// full-batch gather of one layer's halo rows, one tier at a time (used by the epoch's two-stream schedule)
int gather_all_hits(const capgnn_cache *c, int layer, void *out, int64_t ld, hipStream_t st);
int gather_all_misses(const capgnn_cache *c, int layer, void *out, int64_t ld, void *staging, hipStream_t st);
// the two halves of the staged path: DMA of the layer's host tier into the staging area, scatter from there
int stage_misses(const capgnn_cache *c, int layer, void *staging, hipStream_t st);
int scatter_staged(const capgnn_cache *c, int layer, void *out, int64_t ld, void *staging, hipStream_t st);
int gather_hits_and_staged(const capgnn_cache *c, int layer, void *out, int64_t ld, void *staging, hipStream_t st);

}  // namespace capgnn
