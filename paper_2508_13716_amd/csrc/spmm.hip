// Normalised sparse aggregation Y = A_hat X (and, over the CSC, dX = A_hat^T dY) for gfx950.
//
// One 64-wide wavefront owns one output row.  The row's column indices are read 64 at a time,
// one per lane (coalesced), together with the per-entry weight (edge_val * in_scale[col], formed at graph creation); the
// indices are then handed from lane to lane (v_readlane / ds_bpermute) so that every feature-row
// load is a contiguous, 16-byte-per-lane access with a wave-uniform base address.  Several loads
// are kept in flight per wave before any is consumed.  Narrow feature rows (fewer than 64 vectors)
// let a wave work on several edges at once (64/LPR lane groups, combined with a butterfly at the
// end).  Rows with at least LONG_ROW entries are split over the four waves of a workgroup and
// combined through LDS in a fixed order, so results are reproducible run to run.
#include "common.h"

#include <algorithm>

namespace capgnn {

struct SpmmArgs {
    const int64_t *ptr;
    const int32_t *idx;
    const float *out_scale;
    const float *wt;          // per-entry weights, or null: every weight is 1
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
    // cut rows: piece lists and the fp32 partial sums [n_pieces][ldp]
    const int32_t *piece_pos;
    const int32_t *piece_first;
    float *part;
    int64_t ldp;
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

// The same elements kept as loaded (packed bf16 stay packed: half the registers while several loads are in flight)
// and widened only when they are consumed.
template <bool BF16, int E> struct RawVec { float v[E]; };
template <> struct RawVec<true, 8> { uint4 v; };
template <> struct RawVec<true, 1> { uint16_t v; };

template <bool BF16, int E>
__device__ __forceinline__ void load_raw(const char *p, RawVec<BF16, E> &r) {
    if constexpr (BF16 && E == 8) r.v = *reinterpret_cast<const uint4 *>(p);
    else if constexpr (BF16 && E == 1) r.v = *reinterpret_cast<const uint16_t *>(p);
    else load_elems<BF16, E>(p, r.v);
}

template <bool BF16, int E>
__device__ __forceinline__ void zero_raw(RawVec<BF16, E> &r) {
    if constexpr (BF16 && E == 8) r.v = make_uint4(0u, 0u, 0u, 0u);
    else if constexpr (BF16 && E == 1) r.v = 0;
    else {
#pragma unroll
        for (int j = 0; j < E; ++j) r.v[j] = 0.f;
    }
}

template <bool BF16, int E>
__device__ __forceinline__ void fma_raw(float w, const RawVec<BF16, E> &r, float (&acc)[E]) {
    if constexpr (BF16 && E == 8) {
        const uint32_t u[4] = {r.v.x, r.v.y, r.v.z, r.v.w};
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            acc[2 * d] = fmaf(w, __uint_as_float(u[d] << 16), acc[2 * d]);
            acc[2 * d + 1] = fmaf(w, __uint_as_float(u[d] & 0xffff0000u), acc[2 * d + 1]);
        }
    } else if constexpr (BF16 && E == 1) {
        acc[0] = fmaf(w, bf16_bits_to_f32(r.v), acc[0]);
    } else {
#pragma unroll
        for (int j = 0; j < E; ++j) acc[j] = fmaf(w, r.v[j], acc[j]);
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
    } else if constexpr (BF16 && E == 4) {      // float operand, bf16 result: four elements per lane
        uint2 v;
        v.x = f32_to_bf16_bits(x[0]) | (f32_to_bf16_bits(x[1]) << 16);
        v.y = f32_to_bf16_bits(x[2]) | (f32_to_bf16_bits(x[3]) << 16);
        *reinterpret_cast<uint2 *>(p) = v;
    } else {
        static_assert(E == 1, "unsupported element packing");
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
            w = a.wt ? a.wt[my] : 1.f;
        }
        const int cnt = static_cast<int>(e_end - e0 < 64 ? e_end - e0 : 64);
        const int nsteps = (cnt + G - 1) / G;
        int s = 0;
        for (; s + U <= nsteps; s += U) {
            RawVec<BF16, E> x[U][NV];
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
                    if (ok[v]) load_raw<BF16, E>(p + v * LPR * E * ES, x[u][v]);
                    else zero_raw<BF16, E>(x[u][v]);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int v = 0; v < NV; ++v) fma_raw<BF16, E>(ws[u], x[u][v], acc[v]);
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

// The wave-per-row launches are bound by how many gathers the resident waves keep in flight: at least six waves per
// SIMD are asked for (the bf16-in / fp32-out variants otherwise settle at four).
// MODE 0: one single-wave workgroup per output row (rows of one work-list class differ in length, and a wave that
// shares a workgroup with a longer row would hold its slot until that one ends).  MODE 1: one workgroup per row.  MODE 2: one workgroup per piece of a cut row;
// the raw fp32 sum of the piece goes to a.part and spmm_pieces_finish_kernel completes the row.
template <bool BF16, bool OBF16, int E, int LPR, int NV, int MODE>
__global__ __launch_bounds__(MODE == 0 ? 64 : 256, (MODE == 0 && NV < 3) ? 6 : 1) void spmm_kernel(SpmmArgs a) {
    constexpr bool LONG = MODE >= 1;
    constexpr int G = 64 / LPR;
    constexpr int ES = OBF16 ? 2 : 4;   // element size of the output
    constexpr int U = (NV == 1) ? 8 : 4;
    constexpr int PASS = LPR * E * NV;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int l = lane % LPR;
    const int64_t slot = a.list_begin + blockIdx.x;
    if (slot >= a.list_end) return;   // LONG: uniform over the workgroup
    const int row = a.order[MODE == 2 ? a.piece_pos[slot] : slot];
    int64_t beg = a.ptr[row], end = a.ptr[row + 1];
    if constexpr (MODE == 2) {
        beg += static_cast<int64_t>(slot - a.piece_first[a.piece_pos[slot]]) * GIANT_PIECE;
        if (beg + GIANT_PIECE < end) end = beg + GIANT_PIECE;
    }
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
        if constexpr (MODE == 2) {
            if (wave == 0 && lane < LPR) {
                float *prow = a.part + slot * a.ldp;
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    const int f0 = elem0 + v * LPR * E;
#pragma unroll
                    for (int j = 0; j < E; ++j)
                        if (f0 + j < a.F) prow[f0 + j] = acc[v][j];
                }
            }
            continue;
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

// ---------------------------------------------------------------------------------------------------
// Column-blocked variant for dense-degree operators whose gathered matrix is larger than an L2.
//
// A task is (source block cb, output position p, feature slice s): it sums the entries of row order[p] whose
// source lies in block cb, over one SLICE_BYTES-wide slice of the feature row, and stores the partial row to
// scratch.  The grid is laid out so that the workgroups running on one L2 domain at any moment share (cb, s):
// their gathers then address CB_ROWS * SLICE_BYTES = 4 MB, the size of that L2.  Workgroup b runs on domain
// b % NUM_XCD; the slices (times H interleaved shares of the rows when there are fewer slices than domains)
// are dealt to the domains, and each domain sweeps its units block by block.  Within a (unit, block) phase the
// positions come heaviest first in three classes: a whole workgroup per task, a wave per task, and eight
// tasks per wave (one per 8-lane group).  A second kernel sums the partials of a row over the blocks in a
// fixed order and applies the epilogue.
struct SpmmBlockedArgs {
    const uint32_t *off;         // [ncb*n_out + 1]
    const int2 *ew;              // [nnz] {source row, weight bits}
    const uint16_t *src;         // [nnz] source row inside its block: read instead of ew (every weight taken as 1) when not null
    int64_t n_out, n_long, n_mid;
    int ncb, H;                  // source blocks, row shares per slice
    int64_t RG_long, RG_mid, RG; // workgroups per (unit, block): long class, medium class, all
    const char *X;
    uint32_t ld16;               // row pitch of X in 16-byte units
    int F_lim;
    float *part;                 // [ncb*n_out][ldp] partial rows
    int64_t ldp;
};

// entry i of block cb: {source row, weight bits}; from the 2-byte list when the weights are not needed (uniform over
// the launch)
__device__ __forceinline__ int2 blocked_entry(const SpmmBlockedArgs &b, int cb, uint32_t i) {
    return b.src ? make_int2(cb * CB_ROWS + b.src[i], 0x3f800000) : b.ew[i];
}

constexpr int B_LPR = SLICE_BYTES / 16;      // lanes that cover one slice with 16-byte loads
constexpr int B_GROUPS = 64 / B_LPR;         // entries (or rows) a wave works on at the same time
constexpr int B_MID_PER_WAVE = 4;            // consecutive medium positions one wave handles
constexpr int B_SHORT_PER_GROUP = 2;         // consecutive short positions one lane group handles
// entries per trip of a lane group when the entries carry no weights (bf16 rows widen to twice the registers)
template <bool BF16> constexpr int B_SHORT_DEPTH = BF16 ? 8 : 16;
constexpr int B_MID_PER_WG = 4 * B_MID_PER_WAVE;
constexpr int B_SHORT_PER_WG = 4 * B_GROUPS * B_SHORT_PER_GROUP;
static_assert(B_LPR == 8, "lane-group shuffles below assume 8-lane groups");

// value of `v` in lane k of the caller's 8-lane group (ds_swizzle, bit-mask mode: lane = (lane & 0x18) | k)
__device__ __forceinline__ int group_bcast(int v, int k) {
    switch (k) {
        case 0: return __builtin_amdgcn_ds_swizzle(v, 0x0018);
        case 1: return __builtin_amdgcn_ds_swizzle(v, 0x0038);
        case 2: return __builtin_amdgcn_ds_swizzle(v, 0x0058);
        case 3: return __builtin_amdgcn_ds_swizzle(v, 0x0078);
        case 4: return __builtin_amdgcn_ds_swizzle(v, 0x0098);
        case 5: return __builtin_amdgcn_ds_swizzle(v, 0x00b8);
        case 6: return __builtin_amdgcn_ds_swizzle(v, 0x00d8);
        default: return __builtin_amdgcn_ds_swizzle(v, 0x00f8);
    }
}

// All 64 lanes work on ONE row: entries [e0, e1) are read 64 at a time (coalesced), lane group g then takes
// entries g, g+8, ... of the chunk, so up to eight 16-byte-per-lane feature loads are in flight per wave.
// On return every lane of group g holds the sum over that group's entries; the caller adds the groups.
template <bool BF16, bool WEIGHTED, int E>
__device__ __forceinline__ void blocked_row_accumulate(const SpmmBlockedArgs &b, int cb, uint32_t e0, uint32_t e1, int lane,
                                                       const char *xbase, bool ok, float (&acc)[E]) {
    const int grp = lane / B_LPR;
    if constexpr (!WEIGHTED) {
        // bare row numbers: NC chunks of 64 entries per trip (NC * 8 feature loads in flight per lane), plain sums
        // (NC = 2 costs a wave per SIMD in registers and 2 % of the launch: measured)
        constexpr int NC = 1;
        const int rowbase = cb * CB_ROWS;
        int cur[NC];
#pragma unroll
        for (int q = 0; q < NC; ++q) cur[q] = (e0 + 64 * q + lane < e1) ? rowbase + b.src[e0 + 64 * q + lane] : 0;
        for (uint32_t c0 = e0; c0 < e1; c0 += 64 * NC) {
            int coff[NC];
#pragma unroll
            for (int q = 0; q < NC; ++q) coff[q] = static_cast<int>(__umul24(static_cast<uint32_t>(cur[q]), b.ld16));
#pragma unroll
            for (int q = 0; q < NC; ++q)
                cur[q] = (c0 + 64 * (NC + q) + lane < e1) ? rowbase + b.src[c0 + 64 * (NC + q) + lane] : 0;
            const int cnt = static_cast<int>(e1 - c0 < 64u * NC ? e1 - c0 : 64u * NC);
            float xk[NC * B_GROUPS][E];
#pragma unroll
            for (int k = 0; k < NC * B_GROUPS; ++k) {
                const int src = (k % B_GROUPS) * B_GROUPS + grp;             // lane that holds the entry, in chunk k / B_GROUPS
                const uint32_t ck = static_cast<uint32_t>(__shfl(coff[k / B_GROUPS], src));
                if ((k / B_GROUPS) * 64 + src < cnt && ok) {
                    load_elems<BF16, E>(xbase + (static_cast<uint64_t>(ck) << 4), xk[k]);
                } else {
#pragma unroll
                    for (int j = 0; j < E; ++j) xk[k][j] = 0.f;
                }
            }
#pragma unroll
            for (int k = 0; k < NC * B_GROUPS; ++k)
#pragma unroll
                for (int j = 0; j < E; ++j) acc[j] += xk[k][j];
        }
        return;
    }
    int2 pr = make_int2(0, 0);
    if (e0 + lane < e1) pr = blocked_entry(b, cb, e0 + lane);
    for (uint32_t c0 = e0; c0 < e1; c0 += 64) {
        const int coff = static_cast<int>(__umul24(static_cast<uint32_t>(pr.x), b.ld16));   // 16-byte units
        const int wbits = pr.y;                                                               // 0 beyond the end
        pr = make_int2(0, 0);
        if (c0 + 64 + lane < e1) pr = blocked_entry(b, cb, c0 + 64 + lane);      // next chunk's entries are on their way early
        const int cnt = static_cast<int>(e1 - c0 < 64u ? e1 - c0 : 64u);
        float xk[B_GROUPS][E], wk[B_GROUPS];
#pragma unroll
        for (int k = 0; k < B_GROUPS; ++k) {
            if (k * B_GROUPS < cnt) {      // wave-uniform
                const int src = k * B_GROUPS + grp;
                const uint32_t ck = static_cast<uint32_t>(__shfl(coff, src));
                wk[k] = __int_as_float(__shfl(wbits, src));
                if (src < cnt && ok) {
                    load_elems<BF16, E>(xbase + (static_cast<uint64_t>(ck) << 4), xk[k]);
                } else {
#pragma unroll
                    for (int j = 0; j < E; ++j) xk[k][j] = 0.f;
                }
            }
        }
#pragma unroll
        for (int k = 0; k < B_GROUPS; ++k)
            if (k * B_GROUPS < cnt) {
#pragma unroll
                for (int j = 0; j < E; ++j) acc[j] = fmaf(wk[k], xk[k][j], acc[j]);
            }
    }
}

template <int E>
__device__ __forceinline__ void add_groups(float (&acc)[E]) {
#pragma unroll
    for (int off = B_LPR; off < 64; off <<= 1)
#pragma unroll
        for (int j = 0; j < E; ++j) acc[j] += __shfl_xor(acc[j], off);
}

// WEIGHTED: entries come with their weights (b.ew); otherwise as bare block-local row numbers (b.src), every weight 1.
template <bool BF16, bool WEIGHTED>
__global__ __launch_bounds__(256) void spmm_blocked_kernel(SpmmBlockedArgs b) {
    constexpr int E = BF16 ? 8 : 4;
    constexpr int ES = BF16 ? 2 : 4;
    constexpr int SLICE = B_LPR * E;
    __shared__ float red[3][E][B_LPR];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int l = lane % B_LPR, grp = lane / B_LPR;
    const int x = blockIdx.x % NUM_XCD;
    int64_t q = blockIdx.x / NUM_XCD;
    int64_t r = q % b.RG;
    q /= b.RG;
    const int cb = static_cast<int>(q % b.ncb);
    const int64_t u = x + NUM_XCD * (q / b.ncb);     // unit = (slice, share)
    const int s = static_cast<int>(u / b.H), h = static_cast<int>(u % b.H);
    const int elem0 = s * SLICE + l * E;
    const bool ok = elem0 < b.F_lim;
    const char *xbase = b.X + static_cast<int64_t>(elem0) * ES;
    const int64_t tbase = static_cast<int64_t>(cb) * b.n_out;

    if (r < b.RG_long) {
        // ---- a whole workgroup on one task: the four waves take quarters of the group, summed through LDS
        const int64_t p = r * b.H + h;
        if (p >= b.n_long) return;                   // uniform over the workgroup
        const uint32_t e0 = b.off[tbase + p], e1 = b.off[tbase + p + 1];
        if (e0 == e1) return;
        const uint32_t per = ((e1 - e0 + 3) / 4 + 63) / 64 * 64;
        uint32_t w0 = e0 + wave * per, w1 = w0 + per;
        if (w0 > e1) w0 = e1;
        if (w1 > e1) w1 = e1;
        float acc[E];
#pragma unroll
        for (int j = 0; j < E; ++j) acc[j] = 0.f;
        blocked_row_accumulate<BF16, WEIGHTED, E>(b, cb, w0, w1, lane, xbase, ok, acc);
        add_groups<E>(acc);
        if (wave > 0 && lane < B_LPR) {
#pragma unroll
            for (int j = 0; j < E; ++j) red[wave - 1][j][lane] = acc[j];
        }
        __syncthreads();
        if (wave == 0 && lane < B_LPR) {
#pragma unroll
            for (int wv = 0; wv < 3; ++wv)
#pragma unroll
                for (int j = 0; j < E; ++j) acc[j] += red[wv][j][lane];
            store_elems<false, E>(reinterpret_cast<char *>(b.part + (tbase + p) * b.ldp + elem0), acc);
        }
        return;
    }
    r -= b.RG_long;
    if (r < b.RG_mid) {
        // ---- one wave per task
        const int64_t p0 = b.n_long + (r * b.H + h) * B_MID_PER_WG + wave * B_MID_PER_WAVE;
        for (int i = 0; i < B_MID_PER_WAVE; ++i) {
            const int64_t p = p0 + i;
            if (p >= b.n_mid) break;
            const uint32_t e0 = b.off[tbase + p], e1 = b.off[tbase + p + 1];
            if (e0 == e1) continue;
            float acc[E];
#pragma unroll
            for (int j = 0; j < E; ++j) acc[j] = 0.f;
            blocked_row_accumulate<BF16, WEIGHTED, E>(b, cb, e0, e1, lane, xbase, ok, acc);
            add_groups<E>(acc);
            if (lane < B_LPR) store_elems<false, E>(reinterpret_cast<char *>(b.part + (tbase + p) * b.ldp + elem0), acc);
        }
        return;
    }
    r -= b.RG_mid;
    // ---- eight tasks per wave: each 8-lane group owns one position and walks its entries 8 per trip (one index
    // load per group, then 8 independent feature loads in flight)
    const int64_t p0 = b.n_mid + (r * b.H + h) * B_SHORT_PER_WG + wave * (B_GROUPS * B_SHORT_PER_GROUP);
    for (int i = 0; i < B_SHORT_PER_GROUP; ++i) {
        const int64_t p = p0 + i * B_GROUPS + grp;
        uint32_t e = 0, e1 = 0;
        if (p < b.n_out) { e = b.off[tbase + p]; e1 = b.off[tbase + p + 1]; }
        const bool any_entry = e < e1;
        float acc[E];
#pragma unroll
        for (int j = 0; j < E; ++j) acc[j] = 0.f;
        if constexpr (!WEIGHTED) {
            // bare row numbers, B_SHORT_DEPTH entries per trip: each lane fetches an eighth of them, the group exchanges
            // them and every lane has that many feature loads in flight; the sums need no multiply
            constexpr int NQ = B_SHORT_DEPTH<BF16> / B_LPR;
            const int rowbase = cb * CB_ROWS;
            int cur[NQ];
#pragma unroll
            for (int q = 0; q < NQ; ++q) cur[q] = (e + q * B_LPR + l < e1) ? rowbase + b.src[e + q * B_LPR + l] : 0;
            while (__any(e < e1)) {
                const int n = e < e1 ? static_cast<int>(e1 - e) : 0;    // entries this group still has (may exceed a trip)
                int coff[NQ];
#pragma unroll
                for (int q = 0; q < NQ; ++q) coff[q] = static_cast<int>(__umul24(static_cast<uint32_t>(cur[q]), b.ld16));
                e += B_SHORT_DEPTH<BF16>;
#pragma unroll
                for (int q = 0; q < NQ; ++q) cur[q] = (e + q * B_LPR + l < e1) ? rowbase + b.src[e + q * B_LPR + l] : 0;
                float xk[B_SHORT_DEPTH<BF16>][E];
#pragma unroll
                for (int k = 0; k < B_SHORT_DEPTH<BF16>; ++k) {
                    const uint32_t ck = static_cast<uint32_t>(group_bcast(coff[k / B_LPR], k % B_LPR));
                    if (k < n && ok) {
                        load_elems<BF16, E>(xbase + (static_cast<uint64_t>(ck) << 4), xk[k]);
                    } else {
#pragma unroll
                        for (int j = 0; j < E; ++j) xk[k][j] = 0.f;
                    }
                }
#pragma unroll
                for (int k = 0; k < B_SHORT_DEPTH<BF16>; ++k)
#pragma unroll
                    for (int j = 0; j < E; ++j) acc[j] += xk[k][j];
            }
            if (any_entry) store_elems<false, E>(reinterpret_cast<char *>(b.part + (tbase + p) * b.ldp + elem0), acc);
            continue;
        }
        int2 pr = make_int2(0, 0);
        if (e + l < e1) pr = blocked_entry(b, cb, e + l);
        while (__any(e < e1)) {
            const int coff = static_cast<int>(__umul24(static_cast<uint32_t>(pr.x), b.ld16));   // in 16-byte units
            const int wbits = pr.y;
            const int n = e < e1 ? static_cast<int>(e1 - e) : 0;    // entries this group still has (may exceed 8)
            e += B_LPR;
            pr = make_int2(0, 0);
            if (e + l < e1) pr = blocked_entry(b, cb, e + l);                       // next trip's entries are on their way early
            float xk[B_LPR][E], wk[B_LPR];
#pragma unroll
            for (int k = 0; k < B_LPR; ++k) {
                const uint32_t ck = static_cast<uint32_t>(group_bcast(coff, k));
                wk[k] = __int_as_float(group_bcast(wbits, k));
                if (k < n && ok) {
                    load_elems<BF16, E>(xbase + (static_cast<uint64_t>(ck) << 4), xk[k]);
                } else {
#pragma unroll
                    for (int j = 0; j < E; ++j) xk[k][j] = 0.f;
                }
            }
#pragma unroll
            for (int k = 0; k < B_LPR; ++k)
#pragma unroll
                for (int j = 0; j < E; ++j) acc[j] = fmaf(wk[k], xk[k][j], acc[j]);
        }
        if (any_entry) store_elems<false, E>(reinterpret_cast<char *>(b.part + (tbase + p) * b.ldp + elem0), acc);
    }
}

struct SpmmReduceArgs {
    const uint32_t *off;
    const int32_t *order;
    const float *out_scale;
    const float *part;
    int64_t ldp, n_out;
    int ncb;
    char *Y;
    int64_t ldy_bytes;
    int F;
    const float *bias;
    int relu, accumulate;
};

// one thread per (position, four consecutive features)
template <bool OBF16>
__global__ __launch_bounds__(256) void spmm_blocked_reduce_kernel(SpmmReduceArgs a) {
    constexpr int ES = OBF16 ? 2 : 4;
    const int chunks = (a.F + 3) / 4;
    const int64_t tid = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    const int64_t p = tid / chunks;
    if (p >= a.n_out) return;
    const int f0 = static_cast<int>(tid % chunks) * 4;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int cb = 0; cb < a.ncb; ++cb) {
        const int64_t t = static_cast<int64_t>(cb) * a.n_out + p;
        if (a.off[t + 1] == a.off[t]) continue;      // empty group: its partial row was never written
        const float4 v = *reinterpret_cast<const float4 *>(a.part + t * a.ldp + f0);
        acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    const int row = a.order[p];
    const float oscale = a.out_scale ? a.out_scale[row] : 1.f;
    char *yrow = a.Y + static_cast<int64_t>(row) * a.ldy_bytes;
    float y[4] = {acc.x * oscale, acc.y * oscale, acc.z * oscale, acc.w * oscale};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if (f0 + j < a.F) {
            if (a.accumulate) y[j] += load_one<OBF16>(yrow + static_cast<int64_t>(f0 + j) * ES);
            if (a.bias) y[j] += a.bias[f0 + j];
        }
        if (a.relu) y[j] = y[j] > 0.f ? y[j] : 0.f;
    }
    if (f0 + 4 <= a.F) {
        if constexpr (OBF16) {
            uint2 v;
            v.x = f32_to_bf16_bits(y[0]) | (f32_to_bf16_bits(y[1]) << 16);
            v.y = f32_to_bf16_bits(y[2]) | (f32_to_bf16_bits(y[3]) << 16);
            *reinterpret_cast<uint2 *>(yrow + static_cast<int64_t>(f0) * ES) = v;
        } else {
            *reinterpret_cast<float4 *>(yrow + static_cast<int64_t>(f0) * ES) = make_float4(y[0], y[1], y[2], y[3]);
        }
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (f0 + j < a.F) store_one<OBF16>(yrow + static_cast<int64_t>(f0 + j) * ES, y[j]);
    }
}

// Geometry of the blocked launch for a width-F operand; ok == false when the blocked kernel does not apply.
struct BlockedGeom {
    bool ok = false;
    int ns = 0, H = 0;
    int64_t U = 0, RG_long = 0, RG_mid = 0, RG = 0, ldp = 0, grid = 0;
    size_t ws = 0;
};

static BlockedGeom blocked_geom(const SpOp &op, int F, int dtype) {
    BlockedGeom g;
    if (op.ncb == 0 || F <= 0) return g;
    const int slice = SLICE_BYTES / elem_bytes(dtype);
    if (F < slice) return g;                         // narrow rows: the whole operand is small, one pass does
    if (op.n_in >= (int64_t(1) << 24)) return g;     // the kernel forms source offsets with 24-bit multiplies
    g.ns = (F + slice - 1) / slice;
    int gcd = g.ns, t = NUM_XCD;
    while (t) { const int m = gcd % t; gcd = t; t = m; }
    g.H = NUM_XCD / gcd;
    g.U = static_cast<int64_t>(g.ns) * g.H / NUM_XCD;
    auto per_share = [&](int64_t positions, int per_wg) { return ((positions + per_wg - 1) / per_wg + g.H - 1) / g.H; };
    g.RG_long = per_share(op.b_long, 1);
    g.RG_mid = per_share(op.b_mid - op.b_long, B_MID_PER_WG);
    g.RG = g.RG_long + g.RG_mid + per_share(op.n_out - op.b_mid, B_SHORT_PER_WG);
    g.ldp = static_cast<int64_t>(g.ns) * slice;
    g.grid = NUM_XCD * g.U * op.ncb * g.RG;
    if (g.grid <= 0 || g.grid >= (int64_t(1) << 31)) return g;
    g.ws = align_up(static_cast<size_t>(op.ncb) * op.n_out * g.ldp * sizeof(float), 256);
    g.ok = true;
    return g;
}

static int64_t pieces_ldp(int F) { return (static_cast<int64_t>(F) + 7) / 8 * 8; }

size_t spmm_ws_bytes(const SpOp &op, int F, int dtype) {
    const BlockedGeom g = blocked_geom(op, F, dtype);
    const int64_t pieces = std::max(op.giant.n_pieces, op.giant_sub.n_pieces);
    const size_t cut = F > 0 ? static_cast<size_t>(pieces) * pieces_ldp(F) * sizeof(float) : 0;
    return std::max<size_t>(g.ok ? g.ws : 0, cut);
}

template <bool BF16, bool OBF16>
static int launch_blocked(const SpOp &op, const BlockedGeom &g, const SpmmArgs &a, float *part, hipStream_t st) {
    SpmmBlockedArgs b;
    b.off = op.b_off; b.ew = op.b_ew; b.src = (a.wt == nullptr) ? op.b_src : nullptr; b.n_out = op.n_out; b.n_long = op.b_long; b.n_mid = op.b_mid;
    b.ncb = op.ncb; b.H = g.H; b.RG_long = g.RG_long; b.RG_mid = g.RG_mid; b.RG = g.RG;
    b.X = a.X; b.ld16 = static_cast<uint32_t>(a.ldx_bytes >> 4); b.F_lim = a.F_lim;
    b.part = part; b.ldp = g.ldp;
    if (b.src) hipLaunchKernelGGL((spmm_blocked_kernel<BF16, false>), dim3(static_cast<unsigned>(g.grid)), dim3(256), 0, st, b);
    else hipLaunchKernelGGL((spmm_blocked_kernel<BF16, true>), dim3(static_cast<unsigned>(g.grid)), dim3(256), 0, st, b);
    CG_HIP(hipGetLastError());
    SpmmReduceArgs r;
    r.off = op.b_off; r.order = op.order; r.out_scale = op.out_scale; r.part = part; r.ldp = g.ldp; r.n_out = op.n_out;
    r.ncb = op.ncb; r.Y = a.Y; r.ldy_bytes = a.ldy_bytes; r.F = a.F; r.bias = a.bias; r.relu = a.relu;
    r.accumulate = a.accumulate;
    const int64_t threads = op.n_out * ((a.F + 3) / 4);
    hipLaunchKernelGGL((spmm_blocked_reduce_kernel<OBF16>), dim3(static_cast<unsigned>((threads + 255) / 256)), dim3(256),
                       0, st, r);
    CG_HIP(hipGetLastError());
    return CAPGNN_OK;
}

// Completes the cut rows: sums the pieces of a row in piece order and applies the same epilogue as spmm_kernel.
template <bool OBF16>
__global__ __launch_bounds__(256) void spmm_pieces_finish_kernel(SpmmArgs a, int64_t n_giant) {
    constexpr int ES = OBF16 ? 2 : 4;
    const int64_t t = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (t >= n_giant * a.F) return;
    const int64_t pos = t / a.F;
    const int f = static_cast<int>(t - pos * a.F);
    const int row = a.order[pos];
    float acc = 0.f;
    for (int q = a.piece_first[pos]; q < a.piece_first[pos + 1]; ++q) acc += a.part[q * a.ldp + f];
    acc *= a.out_scale ? a.out_scale[row] : 1.f;
    char *y = a.Y + static_cast<int64_t>(row) * a.ldy_bytes + static_cast<int64_t>(f) * ES;
    if (a.accumulate) acc += load_one<OBF16>(y);
    if (a.bias) acc += a.bias[f];
    if (a.relu) acc = acc > 0.f ? acc : 0.f;
    store_one<OBF16>(y, acc);
}

template <bool BF16, bool OBF16, int E, int LPR, int NV>
static int launch_cfg(const SpmmArgs &base, const GiantList *giant, int64_t n_long, int64_t n_rows, hipStream_t st) {
    int64_t n_giant = 0;
    if (giant) {
        n_giant = giant->n_rows;
        SpmmArgs a = base;
        a.list_begin = 0;
        a.list_end = giant->n_pieces;
        hipLaunchKernelGGL((spmm_kernel<BF16, OBF16, E, LPR, NV, 2>), dim3(static_cast<unsigned>(giant->n_pieces)),
                           dim3(256), 0, st, a);
        const int64_t threads = n_giant * a.F;
        hipLaunchKernelGGL((spmm_pieces_finish_kernel<OBF16>), dim3(static_cast<unsigned>((threads + 255) / 256)),
                           dim3(256), 0, st, a, n_giant);
    }
    if (n_long > n_giant) {
        SpmmArgs a = base;
        a.list_begin = n_giant;
        a.list_end = n_long;
        hipLaunchKernelGGL((spmm_kernel<BF16, OBF16, E, LPR, NV, 1>), dim3(static_cast<unsigned>(n_long - n_giant)),
                           dim3(256), 0, st, a);
    }
    if (n_rows > n_long) {
        SpmmArgs a = base;
        a.list_begin = n_long;
        a.list_end = n_rows;
        hipLaunchKernelGGL((spmm_kernel<BF16, OBF16, E, LPR, NV, 0>), dim3(static_cast<unsigned>(n_rows - n_long)),
                           dim3(64), 0, st, a);
    }
    CG_HIP(hipGetLastError());
    return CAPGNN_OK;
}

template <bool BF16, bool OBF16>
static int dispatch(const SpmmArgs &a, bool vec, const GiantList *gl, int64_t n_long, int64_t n_rows, hipStream_t st) {
    constexpr int EV = BF16 ? 8 : 4;
    if (vec) {
        const int nvec = a.F_lim / EV;
        if (nvec <= 4) return launch_cfg<BF16, OBF16, EV, 4, 1>(a, gl, n_long, n_rows, st);
        if (nvec <= 8) return launch_cfg<BF16, OBF16, EV, 8, 1>(a, gl, n_long, n_rows, st);
        if (nvec <= 16) return launch_cfg<BF16, OBF16, EV, 16, 1>(a, gl, n_long, n_rows, st);
        if (nvec <= 32) return launch_cfg<BF16, OBF16, EV, 32, 1>(a, gl, n_long, n_rows, st);
        if (nvec <= 64) return launch_cfg<BF16, OBF16, EV, 64, 1>(a, gl, n_long, n_rows, st);
        if (nvec <= 128) return launch_cfg<BF16, OBF16, EV, 64, 2>(a, gl, n_long, n_rows, st);
        return launch_cfg<BF16, OBF16, EV, 64, 3>(a, gl, n_long, n_rows, st);   // wider rows take several passes
    }
    if (a.F <= 64) return launch_cfg<BF16, OBF16, 1, 64, 1>(a, gl, n_long, n_rows, st);
    if (a.F <= 128) return launch_cfg<BF16, OBF16, 1, 64, 2>(a, gl, n_long, n_rows, st);
    return launch_cfg<BF16, OBF16, 1, 64, 4>(a, gl, n_long, n_rows, st);
}

int launch_spmm(const SpOp &op, bool restrict_sub, const void *X, int64_t ldx, void *Y, int64_t ldy, int F,
                int dtype, const SpmmEpilogue &ep, hipStream_t stream) {
    int out_dtype = (ep.out_f32 || dtype == CAPGNN_F32) ? CAPGNN_F32 : CAPGNN_BF16;
    if (ep.out_bf16 && dtype == CAPGNN_F32) out_dtype = CAPGNN_BF16;     // float operand, rounded once on the way out
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
    a.ptr = op.ptr; a.idx = op.idx; a.out_scale = op.out_scale;
    a.wt = op.wt;
    if (ep.operand_scaled) {
        if (!op.weights_by_source) CG_FAIL(CAPGNN_EINVAL, "spmm: operand_scaled asks for an operator whose weights depend on the source alone");
        a.wt = nullptr;             // the rows of X carry the weights
    }
    a.order = restrict_sub ? op.order_sub : op.order;
    a.list_begin = 0; a.list_end = n_rows;
    a.X = static_cast<const char *>(X); a.ldx_bytes = ldx * es;
    a.Y = static_cast<char *>(Y); a.ldy_bytes = ldy * es_out;
    a.F = F; a.F_lim = vec ? f_up : F;
    a.bias = ep.bias; a.relu = ep.relu; a.accumulate = ep.accumulate;
    const int64_t n_long = restrict_sub ? op.n_long_sub : op.n_long;
    if (vec && !restrict_sub && ep.ws) {
        // the blocked kernel runs when the operator has a blocked copy and the caller brought the scratch for it
        const BlockedGeom bg = blocked_geom(op, F, dtype);
        // source offsets are 32-bit counts of 16-byte units formed by a 24-bit multiply
        const bool off_ok = (a.ldx_bytes >> 4) < (int64_t(1) << 24) && op.n_in * (a.ldx_bytes >> 4) < (int64_t(1) << 32);
        if (bg.ok && off_ok && ep.ws_bytes >= bg.ws && (reinterpret_cast<uintptr_t>(ep.ws) & 15u) == 0) {
            float *part = static_cast<float *>(ep.ws);
            if (dtype == CAPGNN_F32 && out_dtype == CAPGNN_BF16) return launch_blocked<false, true>(op, bg, a, part, stream);
            if (dtype == CAPGNN_F32) return launch_blocked<false, false>(op, bg, a, part, stream);
            if (out_dtype == CAPGNN_BF16) return launch_blocked<true, true>(op, bg, a, part, stream);
            return launch_blocked<true, false>(op, bg, a, part, stream);
        }
    }
    // rows too long for one workgroup are cut into pieces when the caller brought scratch for their partial sums
    const GiantList &gl = restrict_sub ? op.giant_sub : op.giant;
    const GiantList *cut = nullptr;
    a.piece_pos = gl.piece_pos; a.piece_first = gl.piece_first;
    a.part = static_cast<float *>(ep.ws); a.ldp = pieces_ldp(F);
    if (gl.n_rows > 0 && ep.ws && (reinterpret_cast<uintptr_t>(ep.ws) & 15u) == 0 &&
        ep.ws_bytes >= static_cast<size_t>(gl.n_pieces) * a.ldp * sizeof(float))
        cut = &gl;
    if (dtype == CAPGNN_F32 && out_dtype == CAPGNN_BF16) return dispatch<false, true>(a, vec, cut, n_long, n_rows, stream);
    if (dtype == CAPGNN_F32) return dispatch<false, false>(a, vec, cut, n_long, n_rows, stream);
    if (out_dtype == CAPGNN_BF16) return dispatch<true, true>(a, vec, cut, n_long, n_rows, stream);
    return dispatch<true, false>(a, vec, cut, n_long, n_rows, stream);
}

// Measurement aid for the gather roofline: every 8-lane group fetches 128-byte lines (16 bytes per lane) at
// pseudo-random line numbers inside a table, 16 independent loads in flight per lane, nothing else: no index
// stream, no lane exchange, no stores but one checksum per thread.  What it reaches on a table that fits an L2, the
// Infinity Cache, or neither is the rate those levels deliver for this access pattern.
__global__ __launch_bounds__(256) void gather_peak_kernel(const uint4 *table, uint32_t line_mask, uint32_t line_stride, int iters,
                                                          float *out) {
    const uint32_t group = (blockIdx.x * 256u + threadIdx.x) >> 3;
    const uint32_t l = threadIdx.x & 7u;
    const uint4 *base = table + l;
    float acc = 0.f;
    uint32_t x = group * 0x9E3779B1u + 12345u;
    for (int it = 0; it < iters; ++it) {
        uint4 v[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            x = x * 1664525u + 1013904223u;                          // the same sequence in all lanes of a group
            const uint32_t line = (x >> 7) & line_mask;              // the high bits of the generator: the low ones cycle
            v[k] = base[static_cast<uint64_t>(line * line_stride) << 3];
        }
#pragma unroll
        for (int k = 0; k < 16; ++k)      // all four words are consumed, so the load stays one 16-byte access per lane
            acc += __uint_as_float((v[k].x ^ v[k].y ^ v[k].z ^ v[k].w) & 0x3f800000u);
    }
    out[blockIdx.x * 256u + threadIdx.x] = acc;
}

}  // namespace capgnn

using namespace capgnn;

extern "C" int capgnn_gather_peak(const void *table, int64_t table_lines, int line_stride, int workgroups, int iters,
                                  float *out, double *bytes, void *stream) {
    if (!table || table_lines <= 0 || table_lines > (1LL << 24) || (table_lines & (table_lines - 1)) != 0 || workgroups <= 0 ||
        iters <= 0 || !out || !bytes || !aligned16(table) || line_stride < 1 || table_lines * line_stride > (int64_t(1) << 28))
        CG_FAIL(CAPGNN_EINVAL, "gather_peak: bad argument (table_lines must be a power of two, at most 2^24)");
    hipLaunchKernelGGL(gather_peak_kernel, dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4 *>(table), static_cast<uint32_t>(table_lines - 1), static_cast<uint32_t>(line_stride),
                       iters, out);
    CG_HIP(hipGetLastError());
    *bytes = 128.0 * 16.0 * iters * 32.0 * workgroups;      // 32 lane groups per workgroup
    return CAPGNN_OK;
}

extern "C" size_t capgnn_spmm_workspace_bytes(const capgnn_graph *g, int F, int dtype) {
    if (!g || (dtype != CAPGNN_F32 && dtype != CAPGNN_BF16)) return 0;
    return std::max(spmm_ws_bytes(g->fwd, F, dtype), spmm_ws_bytes(g->bwd, F, dtype));
}

extern "C" int capgnn_spmm_fwd(const capgnn_graph *g, const void *X, int64_t ldx, void *Y, int64_t ldy, int F,
                               int dtype, void *ws, size_t ws_bytes, void *stream) {
    if (!g) CG_FAIL(CAPGNN_EINVAL, "spmm_fwd: graph is NULL");
    SpmmEpilogue ep;
    ep.ws = ws; ep.ws_bytes = ws_bytes;
    return launch_spmm(g->fwd, false, X, ldx, Y, ldy, F, dtype, ep, static_cast<hipStream_t>(stream));
}

extern "C" int capgnn_spmm_bwd(const capgnn_graph *g, const void *dY, int64_t lddy, void *dX, int64_t lddx, int F,
                               int dtype, void *ws, size_t ws_bytes, void *stream) {
    if (!g) CG_FAIL(CAPGNN_EINVAL, "spmm_bwd: graph is NULL");
    SpmmEpilogue ep;
    ep.ws = ws; ep.ws_bytes = ws_bytes;
    return launch_spmm(g->bwd, false, dY, lddy, dX, lddx, F, dtype, ep, static_cast<hipStream_t>(stream));
}
