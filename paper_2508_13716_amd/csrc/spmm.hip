// Normalised sparse aggregation Y = A_hat X (and, over the CSC, dX = A_hat^T dY) for gfx950.
//
// One 64-wide wavefront owns one output row.  The row's column indices are read 64 at a time,
// one per lane (coalesced), together with the per-edge weight edge_val * in_scale[col]; the
// indices are then handed from lane to lane (v_readlane / ds_bpermute) so that every feature-row
// load is a contiguous, 16-byte-per-lane access with a wave-uniform base address.  Several loads
// are kept in flight per wave before any is consumed.  Narrow feature rows (fewer than 64 vectors)
// let a wave work on several edges at once (64/LPR lane groups, combined with a butterfly at the
// end).  Rows with at least LONG_ROW entries are split over the four waves of a workgroup and
// combined through LDS in a fixed order, so results are reproducible run to run.
#include "common.h"

namespace capgnn {

struct SpmmArgs {
    const int64_t *ptr;
    const int32_t *idx;
    const float *val;
    const float *out_scale;
    const float *in_scale;
    const int32_t *order;
    int64_t list_begin, list_end;
    const char *X;
    int64_t ldx_bytes;
    char *Y;
    int64_t ldy_bytes;
    int F;        // valid elements per row
    int F_lim;    // elements covered by loads (F rounded up to the vector width)
    const float *bias;
    int relu;
    int accumulate;
};

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;  // quiet NaN
    u += 0x7fffu + ((u >> 16) & 1u);                                   // round to nearest even
    return u >> 16;
}

template <bool BF16, int E>
__device__ __forceinline__ void load_elems(const char *p, float (&x)[E]) {
    if constexpr (!BF16 && E == 4) {
        float4 v = *reinterpret_cast<const float4 *>(p);
        x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
    } else if constexpr (!BF16 && E == 1) {
        x[0] = *reinterpret_cast<const float *>(p);
    } else if constexpr (BF16 && E == 8) {
        uint4 v = *reinterpret_cast<const uint4 *>(p);
        x[0] = __uint_as_float(v.x << 16); x[1] = __uint_as_float(v.x & 0xffff0000u);
        x[2] = __uint_as_float(v.y << 16); x[3] = __uint_as_float(v.y & 0xffff0000u);
        x[4] = __uint_as_float(v.z << 16); x[5] = __uint_as_float(v.z & 0xffff0000u);
        x[6] = __uint_as_float(v.w << 16); x[7] = __uint_as_float(v.w & 0xffff0000u);
    } else {
        static_assert(BF16 && E == 1, "unsupported element packing");
        x[0] = bf16_bits_to_f32(*reinterpret_cast<const uint16_t *>(p));
    }
}

template <bool BF16>
__device__ __forceinline__ float load_one(const char *p) {
    if constexpr (BF16) return bf16_bits_to_f32(*reinterpret_cast<const uint16_t *>(p));
    else return *reinterpret_cast<const float *>(p);
}

template <bool BF16>
__device__ __forceinline__ void store_one(char *p, float v) {
    if constexpr (BF16) *reinterpret_cast<uint16_t *>(p) = static_cast<uint16_t>(f32_to_bf16_bits(v));
    else *reinterpret_cast<float *>(p) = v;
}

template <bool BF16, int E>
__device__ __forceinline__ void store_elems(char *p, const float (&x)[E]) {
    if constexpr (!BF16 && E == 4) {
        *reinterpret_cast<float4 *>(p) = make_float4(x[0], x[1], x[2], x[3]);
    } else if constexpr (!BF16 && E == 8) {
        reinterpret_cast<float4 *>(p)[0] = make_float4(x[0], x[1], x[2], x[3]);
        reinterpret_cast<float4 *>(p)[1] = make_float4(x[4], x[5], x[6], x[7]);
    } else if constexpr (BF16 && E == 8) {
        uint4 v;
        v.x = f32_to_bf16_bits(x[0]) | (f32_to_bf16_bits(x[1]) << 16);
        v.y = f32_to_bf16_bits(x[2]) | (f32_to_bf16_bits(x[3]) << 16);
        v.z = f32_to_bf16_bits(x[4]) | (f32_to_bf16_bits(x[5]) << 16);
        v.w = f32_to_bf16_bits(x[6]) | (f32_to_bf16_bits(x[7]) << 16);
        *reinterpret_cast<uint4 *>(p) = v;
    } else {
        store_one<BF16>(p, x[0]);
    }
}

// Adds, for the entries [e_begin, e_end) of one output row, weight * X[source, lane's features] to acc.
template <bool BF16, int E, int LPR, int NV, int U>
__device__ __forceinline__ void accumulate_range(const SpmmArgs &a, int64_t e_begin, int64_t e_end, int lane,
                                                 int elem0, float (&acc)[NV][E]) {
    constexpr int G = 64 / LPR;
    constexpr int ES = BF16 ? 2 : 4;
    const int sub = lane / LPR;
    const int c_first = a.idx[e_begin];
    bool ok[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) ok[v] = elem0 + v * LPR * E < a.F_lim;
    const char *xbase = a.X + static_cast<int64_t>(elem0) * ES;

    for (int64_t e0 = e_begin; e0 < e_end; e0 += 64) {
        const int64_t my = e0 + lane;
        int c = c_first;
        float w = 0.f;
        if (my < e_end) {
            c = a.idx[my];
            w = a.in_scale ? a.in_scale[c] : 1.f;
            if (a.val) w *= a.val[my];
        }
        const int cnt = static_cast<int>(e_end - e0 < 64 ? e_end - e0 : 64);
        const int nsteps = (cnt + G - 1) / G;
        int s = 0;
        for (; s + U <= nsteps; s += U) {
            float x[U][NV][E];
            float ws[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                int cj;
                if constexpr (G == 1) {
                    cj = __builtin_amdgcn_readlane(c, s + u);
                    ws[u] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(w), s + u));
                } else {
                    cj = __shfl(c, (s + u) * G + sub);
                    ws[u] = __shfl(w, (s + u) * G + sub);
                }
                const char *p = xbase + static_cast<int64_t>(cj) * a.ldx_bytes;
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    if (ok[v]) load_elems<BF16, E>(p + v * LPR * E * ES, x[u][v]);
                    else {
#pragma unroll
                        for (int j = 0; j < E; ++j) x[u][v][j] = 0.f;
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int v = 0; v < NV; ++v)
#pragma unroll
                    for (int j = 0; j < E; ++j) acc[v][j] = fmaf(ws[u], x[u][v][j], acc[v][j]);
        }
        for (; s < nsteps; ++s) {
            int cj;
            float wj;
            if constexpr (G == 1) {
                cj = __builtin_amdgcn_readlane(c, s);
                wj = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(w), s));
            } else {
                cj = __shfl(c, s * G + sub);
                wj = __shfl(w, s * G + sub);
            }
            const char *p = xbase + static_cast<int64_t>(cj) * a.ldx_bytes;
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                if (ok[v]) {
                    float x[E];
                    load_elems<BF16, E>(p + v * LPR * E * ES, x);
#pragma unroll
                    for (int j = 0; j < E; ++j) acc[v][j] = fmaf(wj, x[j], acc[v][j]);
                }
            }
        }
    }
}

template <bool BF16, bool OBF16, int E, int LPR, int NV, bool LONG>
__global__ __launch_bounds__(256) void spmm_kernel(SpmmArgs a) {
    constexpr int G = 64 / LPR;
    constexpr int ES = OBF16 ? 2 : 4;   // element size of the output
    constexpr int U = (NV == 1) ? 8 : 4;
    constexpr int PASS = LPR * E * NV;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int l = lane % LPR;
    const int64_t slot = a.list_begin + (LONG ? static_cast<int64_t>(blockIdx.x)
                                              : static_cast<int64_t>(blockIdx.x) * 4 + wave);
    if (slot >= a.list_end) return;   // LONG: uniform over the workgroup
    const int row = a.order[slot];
    int64_t beg = a.ptr[row], end = a.ptr[row + 1];
    if constexpr (LONG) {
        const int64_t len = end - beg;
        const int64_t per = ((len + 3) / 4 + 63) / 64 * 64;
        beg = beg + wave * per;
        if (beg > end) beg = end;
        if (beg + per < end) end = beg + per;
    }
    __shared__ float red[LONG ? 3 : 1][NV * E][64];
    const float oscale = a.out_scale ? a.out_scale[row] : 1.f;

    for (int pass = 0; pass < a.F_lim; pass += PASS) {
        const int elem0 = pass + l * E;
        float acc[NV][E];
#pragma unroll
        for (int v = 0; v < NV; ++v)
#pragma unroll
            for (int j = 0; j < E; ++j) acc[v][j] = 0.f;
        if (beg < end) accumulate_range<BF16, E, LPR, NV, U>(a, beg, end, lane, elem0, acc);
        if constexpr (G > 1) {
#pragma unroll
            for (int off = LPR; off < 64; off <<= 1)
#pragma unroll
                for (int v = 0; v < NV; ++v)
#pragma unroll
                    for (int j = 0; j < E; ++j) acc[v][j] += __shfl_xor(acc[v][j], off);
        }
        if constexpr (LONG) {
            if (pass > 0) __syncthreads();
            if (wave > 0) {
#pragma unroll
                for (int v = 0; v < NV; ++v)
#pragma unroll
                    for (int j = 0; j < E; ++j) red[wave - 1][v * E + j][lane] = acc[v][j];
            }
            __syncthreads();
            if (wave == 0) {
#pragma unroll
                for (int wv = 0; wv < 3; ++wv)
#pragma unroll
                    for (int v = 0; v < NV; ++v)
#pragma unroll
                        for (int j = 0; j < E; ++j) acc[v][j] += red[wv][v * E + j][lane];
            }
        }
        if ((!LONG || wave == 0) && lane < LPR) {
            char *yrow = a.Y + static_cast<int64_t>(row) * a.ldy_bytes;
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const int f0 = elem0 + v * LPR * E;
                if (f0 >= a.F) continue;
                float y[E];
#pragma unroll
                for (int j = 0; j < E; ++j) {
                    float t = acc[v][j] * oscale;
                    if (f0 + j < a.F) {
                        if (a.accumulate) t += load_one<OBF16>(yrow + static_cast<int64_t>(f0 + j) * ES);
                        if (a.bias) t += a.bias[f0 + j];
                    }
                    if (a.relu) t = t > 0.f ? t : 0.f;
                    y[j] = t;
                }
                if (f0 + E <= a.F) {
                    store_elems<OBF16, E>(yrow + static_cast<int64_t>(f0) * ES, y);
                } else {
#pragma unroll
                    for (int j = 0; j < E; ++j)
                        if (f0 + j < a.F) store_one<OBF16>(yrow + static_cast<int64_t>(f0 + j) * ES, y[j]);
                }
            }
        }
    }
}

template <bool BF16, bool OBF16, int E, int LPR, int NV>
static int launch_cfg(const SpmmArgs &base, int64_t n_long, int64_t n_rows, hipStream_t st) {
    if (n_long > 0) {
        SpmmArgs a = base;
        a.list_begin = 0;
        a.list_end = n_long;
        hipLaunchKernelGGL((spmm_kernel<BF16, OBF16, E, LPR, NV, true>), dim3(static_cast<unsigned>(n_long)), dim3(256), 0,
                           st, a);
    }
    if (n_rows > n_long) {
        SpmmArgs a = base;
        a.list_begin = n_long;
        a.list_end = n_rows;
        const int64_t blocks = (n_rows - n_long + 3) / 4;
        hipLaunchKernelGGL((spmm_kernel<BF16, OBF16, E, LPR, NV, false>), dim3(static_cast<unsigned>(blocks)), dim3(256), 0,
                           st, a);
    }
    CG_HIP(hipGetLastError());
    return CAPGNN_OK;
}

template <bool BF16, bool OBF16>
static int dispatch(const SpmmArgs &a, bool vec, int64_t n_long, int64_t n_rows, hipStream_t st) {
    constexpr int EV = BF16 ? 8 : 4;
    if (vec) {
        const int nvec = a.F_lim / EV;
        if (nvec <= 4) return launch_cfg<BF16, OBF16, EV, 4, 1>(a, n_long, n_rows, st);
        if (nvec <= 8) return launch_cfg<BF16, OBF16, EV, 8, 1>(a, n_long, n_rows, st);
        if (nvec <= 16) return launch_cfg<BF16, OBF16, EV, 16, 1>(a, n_long, n_rows, st);
        if (nvec <= 32) return launch_cfg<BF16, OBF16, EV, 32, 1>(a, n_long, n_rows, st);
        if (nvec <= 64) return launch_cfg<BF16, OBF16, EV, 64, 1>(a, n_long, n_rows, st);
        if (nvec <= 128) return launch_cfg<BF16, OBF16, EV, 64, 2>(a, n_long, n_rows, st);
        return launch_cfg<BF16, OBF16, EV, 64, 3>(a, n_long, n_rows, st);   // wider rows take several passes
    }
    if (a.F <= 64) return launch_cfg<BF16, OBF16, 1, 64, 1>(a, n_long, n_rows, st);
    if (a.F <= 128) return launch_cfg<BF16, OBF16, 1, 64, 2>(a, n_long, n_rows, st);
    return launch_cfg<BF16, OBF16, 1, 64, 4>(a, n_long, n_rows, st);
}

int launch_spmm(const SpOp &op, bool restrict_sub, const void *X, int64_t ldx, void *Y, int64_t ldy, int F,
                int dtype, const SpmmEpilogue &ep, hipStream_t stream) {
    const int out_dtype = (ep.out_f32 || dtype == CAPGNN_F32) ? CAPGNN_F32 : CAPGNN_BF16;
    if (dtype != CAPGNN_F32 && dtype != CAPGNN_BF16) CG_FAIL(CAPGNN_EINVAL, "spmm: unknown dtype %d", dtype);
    if (F <= 0 || F > (1 << 20)) CG_FAIL(CAPGNN_EINVAL, "spmm: F=%d out of range", F);
    if (ldx < F || ldy < F) CG_FAIL(CAPGNN_EINVAL, "spmm: leading dimension smaller than F");
    const int64_t n_rows = restrict_sub ? op.n_sub : op.n_out;
    if (n_rows == 0) return CAPGNN_OK;
    if (!X || !Y) CG_FAIL(CAPGNN_EINVAL, "spmm: NULL operand");
    const int es = elem_bytes(dtype);
    const int ev = 16 / es;
    const int f_up = (F + ev - 1) / ev * ev;
    const int es_out = elem_bytes(out_dtype);
    const bool vec = aligned16(X) && aligned16(Y) && (ldx * es) % 16 == 0 && (ldy * es_out) % 16 == 0 && ldx >= f_up;
    SpmmArgs a;
    a.ptr = op.ptr; a.idx = op.idx; a.val = op.val; a.out_scale = op.out_scale; a.in_scale = op.in_scale;
    a.order = restrict_sub ? op.order_sub : op.order;
    a.list_begin = 0; a.list_end = n_rows;
    a.X = static_cast<const char *>(X); a.ldx_bytes = ldx * es;
    a.Y = static_cast<char *>(Y); a.ldy_bytes = ldy * es_out;
    a.F = F; a.F_lim = vec ? f_up : F;
    a.bias = ep.bias; a.relu = ep.relu; a.accumulate = ep.accumulate;
    const int64_t n_long = restrict_sub ? op.n_long_sub : op.n_long;
    if (dtype == CAPGNN_F32) return dispatch<false, false>(a, vec, n_long, n_rows, stream);
    if (out_dtype == CAPGNN_BF16) return dispatch<true, true>(a, vec, n_long, n_rows, stream);
    return dispatch<true, false>(a, vec, n_long, n_rows, stream);
}

}  // namespace capgnn

using namespace capgnn;

extern "C" size_t capgnn_spmm_workspace_bytes(const capgnn_graph *, int, int) { return 0; }

extern "C" int capgnn_spmm_fwd(const capgnn_graph *g, const void *X, int64_t ldx, void *Y, int64_t ldy, int F,
                               int dtype, void *, size_t, void *stream) {
    if (!g) CG_FAIL(CAPGNN_EINVAL, "spmm_fwd: graph is NULL");
    return launch_spmm(g->fwd, false, X, ldx, Y, ldy, F, dtype, SpmmEpilogue(), static_cast<hipStream_t>(stream));
}

extern "C" int capgnn_spmm_bwd(const capgnn_graph *g, const void *dY, int64_t lddy, void *dX, int64_t lddx, int F,
                               int dtype, void *, size_t, void *stream) {
    if (!g) CG_FAIL(CAPGNN_EINVAL, "spmm_bwd: graph is NULL");
    return launch_spmm(g->bwd, false, dY, lddy, dX, lddx, F, dtype, SpmmEpilogue(), static_cast<hipStream_t>(stream));
}
