// Dense products on the gfx950 matrix cores: C[M x N] (+)= op(A) op(B), fp32 accumulation.
//
// A workgroup of four 64-wide waves (2 x 2) owns a BM x BN tile of C.  Operand tiles of depth
// BK = 16 are staged through LDS in k-major order (As[k][i], Bs[k][j]) so that the operands of
// v_mfma_f32_32x32x2_f32 (lane l supplies A[i = l%32][k = l/32] and B[k = l/32][j = l%32]) are read
// from consecutive LDS words.  Global loads of the next tile are issued before the MFMAs of the
// current one (register prefetch + two LDS buffers, one barrier per k-step).  bf16 operands are
// widened to fp32 while they are staged.  The vertex-dimension reduction of the weight gradient
// (trans_a) is split over workgroups; partial tiles go to the workspace and are summed in a fixed
// order by a second kernel, which also applies the epilogue.
#include "common.h"

#include <algorithm>
#include <atomic>
#include <type_traits>

namespace capgnn {

typedef float floatx16 __attribute__((ext_vector_type(16)));

struct GemmArgs {
    int64_t M, N, K;
    const char *A; int64_t lda;
    const char *B; int64_t ldb;
    char *C; int64_t ldc;           // final destination
    float *part;                    // split partials [S][M][N] or null
    int64_t k_chunk;                // reduction range per grid.z
    int a_vec, b_vec;               // operand rows allow 4-element vector loads
    int out_bf16, accumulate, relu;
    const float *bias;
    const char *mask; int64_t ldm; int mask_bf16;
    int gx, gy, S;                  // tiles along N, along M, reduction splits
    int c_staged;                   // bf16 kernel: write C through LDS in 16-byte pieces (no mask / accumulate / split)
    const float *rscale;            // C[i,:] *= rscale[i] after everything else (fp32 C), or null
    // two products into one result, C = A W + A2 W2 (gemm_split_kernel<..., DUAL>): the reduction index runs over A's K1
    // columns, padded to K1p (whole steps), and then over A2's K - K1p columns; the cut weights lie one after the other
    const char *A2; int64_t lda2;
    int64_t K1, K1p;
};

// Tile of a workgroup in the one-dimensional grid.  Workgroup b runs on L2 domain b % NUM_XCD; the order is
// chosen so that workgroups that read the same operand data share a domain and follow one another there: the
// tiles of one reduction split (they read the same slab of both operands), or the tiles along N of one row
// block (they read the same rows of A).  Returns false for the padding workgroups at the end of the grid.
__device__ __forceinline__ bool tile_coords(const GemmArgs &g, int *bx, int *by, int *bz) {
    const int64_t b = blockIdx.x;
    const int xcd = static_cast<int>(b % NUM_XCD);
    const int64_t seq = b / NUM_XCD;
    if (g.S > 1) {
        const int64_t tiles = static_cast<int64_t>(g.gx) * g.gy;
        const int64_t z = (seq / tiles) * NUM_XCD + xcd;
        const int64_t t = seq % tiles;
        *bz = static_cast<int>(z); *bx = static_cast<int>(t % g.gx); *by = static_cast<int>(t / g.gx);
        return z < g.S;
    }
    *bz = 0;
    *bx = static_cast<int>(seq % g.gx);
    const int64_t y = (seq / g.gx) * NUM_XCD + xcd;
    *by = static_cast<int>(y);
    return y < g.gy;
}

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

// four consecutive elements starting at element index `off` of a row; only the first nvalid are read
template <bool BF16>
__device__ __forceinline__ float4 load4(const char *base, int64_t off, int nvalid, int vec) {
    float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
    if (nvalid <= 0) return r;
    if constexpr (BF16) {
        const uint16_t *p = reinterpret_cast<const uint16_t *>(base) + off;
        if (vec && nvalid >= 4) {
            uint2 v = *reinterpret_cast<const uint2 *>(p);
            r.x = __uint_as_float(v.x << 16); r.y = __uint_as_float(v.x & 0xffff0000u);
            r.z = __uint_as_float(v.y << 16); r.w = __uint_as_float(v.y & 0xffff0000u);
        } else {
            r.x = __uint_as_float(static_cast<uint32_t>(p[0]) << 16);
            if (nvalid > 1) r.y = __uint_as_float(static_cast<uint32_t>(p[1]) << 16);
            if (nvalid > 2) r.z = __uint_as_float(static_cast<uint32_t>(p[2]) << 16);
            if (nvalid > 3) r.w = __uint_as_float(static_cast<uint32_t>(p[3]) << 16);
        }
    } else {
        const float *p = reinterpret_cast<const float *>(base) + off;
        if (vec && nvalid >= 4) {
            r = *reinterpret_cast<const float4 *>(p);
        } else {
            r.x = p[0];
            if (nvalid > 1) r.y = p[1];
            if (nvalid > 2) r.z = p[2];
            if (nvalid > 3) r.w = p[3];
        }
    }
    return r;
}

// Writes one wave's TM x TN grid of 32x32 accumulator tiles (top-left corner (row0, col0)) with the epilogue.
// D layout of the 32x32 MFMAs: register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32.
template <int TM, int TN>
__device__ __forceinline__ void store_tile(const GemmArgs &g, const floatx16 (&acc)[TM][TN], int64_t row0, int64_t col0,
                                           int l32, int half, int bz) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int64_t col = col0 + j * 32 + l32;
            if (col >= g.N) continue;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = row0 + i * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
                if (row >= g.M) continue;
                float v = acc[i][j][r];
                if (g.part) {
                    g.part[(static_cast<int64_t>(bz) * g.M + row) * g.N + col] = v;
                    continue;
                }
                if (g.accumulate) {
                    v += g.out_bf16 ? __uint_as_float(static_cast<uint32_t>(reinterpret_cast<const uint16_t *>(g.C)[row * g.ldc + col]) << 16)
                                    : reinterpret_cast<const float *>(g.C)[row * g.ldc + col];
                }
                if (g.bias) v += g.bias[col];
                if (g.relu) v = v > 0.f ? v : 0.f;
                if (g.mask) {
                    const float mv = g.mask_bf16 ? __uint_as_float(static_cast<uint32_t>(reinterpret_cast<const uint16_t *>(g.mask)[row * g.ldm + col]) << 16)
                                                 : reinterpret_cast<const float *>(g.mask)[row * g.ldm + col];
                    if (!(mv > 0.f)) v = 0.f;
                }
                if (g.rscale) v *= g.rscale[row];
                if (g.out_bf16) reinterpret_cast<uint16_t *>(g.C)[row * g.ldc + col] = static_cast<uint16_t>(f32_to_bf16_rne(v));
                else reinterpret_cast<float *>(g.C)[row * g.ldc + col] = v;
            }
        }
}

// The same through LDS: a wave rounds 32 rows of its accumulators at a time into a private LDS area (lds, STAGE_BYTES
// per wave) and leaves along the rows of C, 16 bytes per lane, so that a store instruction covers 4 rows x 256 bytes
// instead of 2 x 128 and the read-modify-write of an accumulating product moves whole vectors.  fp32 results only.
template <int TN> constexpr int STAGE_PITCH_T = TN * 32 + 8;  // floats per staged row (four rows further = other half of the banks)
template <int TN> constexpr int STAGE_BYTES_T = 32 * STAGE_PITCH_T<TN> * 4;   // per wave
constexpr int STAGE_BYTES = STAGE_BYTES_T<2>;

// TN: 32-column accumulator tiles side by side in the wave's part (2 or 1)
template <int TN>
__device__ __forceinline__ void store_tile_staged(const GemmArgs &g, const floatx16 (&acc)[2][TN], float *lds, int64_t row0,
                                                  int64_t col0, int lane, int bz) {
    constexpr int STAGE_PITCH = STAGE_PITCH_T<TN>;
    constexpr int CGS = TN * 8;                              // groups of four columns in a row
    constexpr int RPP = 64 / CGS;                            // rows per pass of the wave
    const int l32 = lane & 31, half = lane >> 5;
    float *dst = g.part ? g.part + static_cast<int64_t>(bz) * g.M * g.N : reinterpret_cast<float *>(g.C);
    const int64_t ld = g.part ? g.N : g.ldc;
    const bool vec = (reinterpret_cast<uintptr_t>(dst) % 16 == 0) && (ld % 4 == 0);
    const bool plain = g.part != nullptr;                   // partials take no epilogue
    const int cg = lane % CGS, rq = lane / CGS;             // the lane's column group (4 columns) and row within a pass
    const int64_t col = col0 + 4 * cg;
    float bv[4] = {0.f, 0.f, 0.f, 0.f};
    if (!plain && g.bias)
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (col + e < g.N) bv[e] = g.bias[col + e];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) lds[(8 * (r >> 2) + 4 * half + (r & 3)) * STAGE_PITCH + j * 32 + l32] = acc[i][j][r];
        __builtin_amdgcn_wave_barrier();
        if (col < g.N) {
#pragma unroll
            for (int t = 0; t < 32 / RPP; ++t) {
                const int lr = RPP * t + rq;
                const int64_t row = row0 + i * 32 + lr;
                if (row >= g.M) continue;
                const float4 v4 = *reinterpret_cast<const float4 *>(&lds[lr * STAGE_PITCH + 4 * cg]);
                float v[4] = {v4.x, v4.y, v4.z, v4.w};
                float *out = dst + row * ld + col;
                const bool whole = vec && col + 4 <= g.N;
                if (!plain) {
                    if (g.accumulate) {
                        if (whole) {
                            const float4 c4 = *reinterpret_cast<const float4 *>(out);
                            v[0] += c4.x; v[1] += c4.y; v[2] += c4.z; v[3] += c4.w;
                        } else {
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                if (col + e < g.N) v[e] += out[e];
                        }
                    }
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        v[e] += bv[e];
                        if (g.relu) v[e] = v[e] > 0.f ? v[e] : 0.f;
                    }
                    if (g.mask) {
                        const float *mk = reinterpret_cast<const float *>(g.mask) + row * g.ldm + col;
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (col + e < g.N && !(mk[e] > 0.f)) v[e] = 0.f;
                    }
                    if (g.rscale) {
                        const float rs = g.rscale[row];
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] *= rs;
                    }
                }
                if (whole) {
                    *reinterpret_cast<float4 *>(out) = make_float4(v[0], v[1], v[2], v[3]);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (col + e < g.N) out[e] = v[e];
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
}

constexpr int BK = 16;
constexpr int PAD = 4;

// Stages one operand tile.  KC: the operand is stored with the reduction index contiguous
// (rows = output index); otherwise the output index is contiguous (rows = reduction index).
template <bool BF16, bool KC, int BT>
struct TileLoader {
    static constexpr int NLD = BT * BK / 4 / 256;   // float4 per thread
    float4 r[NLD];

    __device__ __forceinline__ void fetch(const char *base, int64_t ld, int64_t t0, int64_t T, int64_t k0,
                                          int64_t k_end, int vec, int tid) {
#pragma unroll
        for (int q = 0; q < NLD; ++q) {
            const int idx = tid + 256 * q;
            if constexpr (KC) {
                const int row = idx >> 2, kq = idx & 3;
                const int64_t t = t0 + row, k = k0 + 4 * kq;
                const int nv = (t < T) ? static_cast<int>(k_end - k < 4 ? k_end - k : 4) : 0;
                r[q] = load4<BF16>(base, t * ld + k, nv, vec);
            } else {
                constexpr int QPR = BT / 4;
                const int kk = idx / QPR, tq = idx % QPR;
                const int64_t k = k0 + kk, t = t0 + 4 * tq;
                const int nv = (k < k_end) ? static_cast<int>(T - t < 4 ? T - t : 4) : 0;
                r[q] = load4<BF16>(base, k * ld + t, nv, vec);
            }
        }
    }

    // Interior tiles (every row of the tile exists, vector loads allowed) skip all range checks: the address of
    // each of the thread's vectors is formed once and then only stepped along the reduction index.
    const char *pf[NLD];

    __device__ __forceinline__ void fast_begin(const char *base, int64_t ld, int64_t t0, int64_t k0, int tid) {
        constexpr int ES = BF16 ? 2 : 4;
#pragma unroll
        for (int q = 0; q < NLD; ++q) {
            const int idx = tid + 256 * q;
            if constexpr (KC) pf[q] = base + ((t0 + (idx >> 2)) * ld + k0 + 4 * (idx & 3)) * ES;
            else pf[q] = base + ((k0 + idx / (BT / 4)) * ld + t0 + 4 * (idx % (BT / 4))) * ES;
        }
    }

    __device__ __forceinline__ void fetch_fast(int64_t ld) {
        constexpr int ES = BF16 ? 2 : 4;
        const int64_t step = KC ? static_cast<int64_t>(BK) * ES : static_cast<int64_t>(BK) * ld * ES;
#pragma unroll
        for (int q = 0; q < NLD; ++q) {
            if constexpr (BF16) {
                const uint2 v = *reinterpret_cast<const uint2 *>(pf[q]);
                r[q] = make_float4(__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xffff0000u),
                                   __uint_as_float(v.y << 16), __uint_as_float(v.y & 0xffff0000u));
            } else {
                r[q] = *reinterpret_cast<const float4 *>(pf[q]);
            }
            pf[q] += step;
        }
    }

    __device__ __forceinline__ void stash(float (*s)[BT + PAD], int tid) const {
#pragma unroll
        for (int q = 0; q < NLD; ++q) {
            const int idx = tid + 256 * q;
            if constexpr (KC) {
                const int row = idx >> 2, kq = idx & 3;
                s[4 * kq + 0][row] = r[q].x;
                s[4 * kq + 1][row] = r[q].y;
                s[4 * kq + 2][row] = r[q].z;
                s[4 * kq + 3][row] = r[q].w;
            } else {
                constexpr int QPR = BT / 4;
                const int kk = idx / QPR, tq = idx % QPR;
                *reinterpret_cast<float4 *>(&s[kk][4 * tq]) = r[q];
            }
        }
    }
};

template <bool BF16, bool A_KC, bool B_KC, int BM, int BN>
__global__ __launch_bounds__(256) void gemm_kernel(GemmArgs g) {
    constexpr int WM = BM / 2, WN = BN / 2;
    constexpr int TM = WM / 32, TN = WN / 32;
    // operand tiles; fp32 results of full-size tiles leave through the same memory (store_tile_staged)
    constexpr int OPERAND_FLOATS = 2 * BK * (BM + PAD) + 2 * BK * (BN + PAD);
    constexpr bool STAGED = !BF16 && TM == 2 && TN == 2;
    constexpr int SMEM_FLOATS = (STAGED && 4 * STAGE_BYTES / 4 > OPERAND_FLOATS) ? 4 * STAGE_BYTES / 4 : OPERAND_FLOATS;
    __shared__ __attribute__((aligned(16))) float smem[SMEM_FLOATS];
    float (*As)[BK][BM + PAD] = reinterpret_cast<float (*)[BK][BM + PAD]>(smem);
    float (*Bs)[BK][BN + PAD] = reinterpret_cast<float (*)[BK][BN + PAD]>(smem + 2 * BK * (BM + PAD));

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, half = lane >> 5;
    int bx, by, bz;
    if (!tile_coords(g, &bx, &by, &bz)) return;      // uniform over the workgroup
    const int64_t m0 = static_cast<int64_t>(by) * BM;
    const int64_t n0 = static_cast<int64_t>(bx) * BN;
    const int64_t k_begin = static_cast<int64_t>(bz) * g.k_chunk;
    const int64_t k_end = (k_begin + g.k_chunk < g.K) ? k_begin + g.k_chunk : g.K;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    TileLoader<BF16, A_KC, BM> la;
    TileLoader<BF16, B_KC, BN> lb;
    const int64_t nk = (k_end > k_begin) ? (k_end - k_begin + BK - 1) / BK : 0;
    // uniform over the workgroup: the tile lies inside the matrices and both operands allow vector loads (measured
    // to pay only when the first operand is stored along the reduction index; X^T G keeps the checked loads)
    const bool interior = A_KC && m0 + BM <= g.M && n0 + BN <= g.N && g.a_vec && g.b_vec;
    const int64_t nk_full = (k_end > k_begin) ? (k_end - k_begin) / BK : 0;     // steps that need no check along k either
    if (nk > 0) {
        la.fetch(g.A, g.lda, m0, g.M, k_begin, k_end, g.a_vec, tid);
        lb.fetch(g.B, g.ldb, n0, g.N, k_begin, k_end, g.b_vec, tid);
        la.stash(As[0], tid);
        lb.stash(Bs[0], tid);
    }
    if (interior) {
        la.fast_begin(g.A, g.lda, m0, k_begin + BK, tid);
        lb.fast_begin(g.B, g.ldb, n0, k_begin + BK, tid);
    }
    __syncthreads();
    for (int64_t kt = 0; kt < nk; ++kt) {
        const int buf = static_cast<int>(kt & 1);
        const bool more = kt + 1 < nk;
        if (more) {
            if (interior && kt + 1 < nk_full) {
                la.fetch_fast(g.lda);
                lb.fetch_fast(g.ldb);
            } else {
                la.fetch(g.A, g.lda, m0, g.M, k_begin + (kt + 1) * BK, k_end, g.a_vec, tid);
                lb.fetch(g.B, g.ldb, n0, g.N, k_begin + (kt + 1) * BK, k_end, g.b_vec, tid);
            }
        }
        // operands of step kk+2 are read from LDS before the products of step kk are issued
        float a[2][TM], b[2][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) a[0][i] = As[buf][half][wm * WM + i * 32 + l32];
#pragma unroll
        for (int j = 0; j < TN; ++j) b[0][j] = Bs[buf][half][wn * WN + j * 32 + l32];
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
#pragma unroll
        for (int kk = 0; kk < BK; kk += 2) {
            const int cur = (kk >> 1) & 1;
            if (kk + 2 < BK) {
#pragma unroll
                for (int i = 0; i < TM; ++i) a[cur ^ 1][i] = As[buf][kk + 2 + half][wm * WM + i * 32 + l32];
#pragma unroll
                for (int j = 0; j < TN; ++j) b[cur ^ 1][j] = Bs[buf][kk + 2 + half][wn * WN + j * 32 + l32];
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[cur][i], b[cur][j], acc[i][j], 0, 0, 0);
            // keep that order in the schedule: LDS reads of the next step, then this step's matrix instructions
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, TM * TN, 0);
        }
        if (more) {
            la.stash(As[buf ^ 1], tid);
            lb.stash(Bs[buf ^ 1], tid);
        }
        __syncthreads();
    }

    if constexpr (STAGED) {
        // the last pass through the loop ended with a barrier: every wave is done with the operands
        store_tile_staged(g, acc, smem + wave * (STAGE_BYTES / 4), m0 + wm * WM, n0 + wn * WN, lane, bz);
    } else {
        store_tile<TM, TN>(g, acc, m0 + wm * WM, n0 + wn * WN, l32, half, bz);
    }
}

// ---------------------------------------------------------------------------------------------------
// bf16 operands on the bf16 matrix cores (v_mfma_f32_32x32x16_bf16: lane l supplies A[i = l%32][k = 8*(l/32) ..+7]
// and B[k = 8*(l/32) ..+7][j = l%32], eight consecutive k per lane).  Both operand tiles are kept in LDS with
// the reduction index contiguous (S[row][k], 32 k per step = four 16-byte chunks, rows padded to 80 bytes; the
// chunk position is XOR-ed with bits of the row so that neither the operand reads nor the transposing stores pile
// up on a few banks).  An operand stored with the reduction index contiguous is moved with 16-byte loads and
// stores.  One stored the other way (the vertex dimension of the weight gradient X^T G) is loaded 16 bytes along
// its rows, four consecutive k per thread, transposed in registers (byte permutes pair up the values of two k)
// and stored as 8-byte pieces: no 2-byte LDS traffic.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
constexpr int HBK = 32;            // k per step of the bf16 kernel
constexpr int HPAD = 8;            // bf16 elements of row padding

// position (in elements) of 16-byte chunk `chunk` (0..3) inside LDS row `row`
__device__ __forceinline__ int chunk_pos(int row, int chunk) { return 8 * (chunk ^ ((row >> 3) & 3)); }

// TOFF: first thread of the workgroup that works on this tile when the operand needs the transposing path
// (that path keeps (HBK/4) * (BT/8) threads busy; the two operands of X^T G take disjoint thread ranges).
template <bool KC, int BT, int TOFF>
struct HalfTileLoader {
    static constexpr int NLD = KC ? BT * HBK / 8 / 256 : 4;   // 16-byte chunks per thread
    static constexpr int NTH = (HBK / 4) * (BT / 8);          // threads of the transposing path
    uint4 r[NLD];

    // eight consecutive bf16 starting at element `off`; only the first nvalid are read
    static __device__ __forceinline__ uint4 load8(const char *base, int64_t off, int nvalid) {
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (nvalid <= 0) return v;
        const uint16_t *p = reinterpret_cast<const uint16_t *>(base) + off;
        if (nvalid >= 8) return *reinterpret_cast<const uint4 *>(p);
        uint32_t w[4] = {0u, 0u, 0u, 0u};
        for (int e = 0; e < nvalid; ++e) w[e >> 1] |= static_cast<uint32_t>(p[e]) << (16 * (e & 1));
        return make_uint4(w[0], w[1], w[2], w[3]);
    }

    int64_t k_rows = 0;             // rows of the operand when it is stored across the reduction index (set by the kernel)

    __device__ __forceinline__ void fetch(const char *base, int64_t ld, int64_t t0, int64_t T, int64_t k0, int64_t k_end,
                                          int tid) {
        if constexpr (KC) {
#pragma unroll
            for (int q = 0; q < NLD; ++q) {
                const int idx = tid + 256 * q;
                const int row = idx >> 2, kq = idx & 3;
                const int64_t t = t0 + row, k = k0 + 8 * kq;
                const int nv = (t < T) ? static_cast<int>(k_end - k < 8 ? k_end - k : 8) : 0;
                r[q] = load8(base, t * ld + k, nv);
            }
        } else {
            const int tt = tid - TOFF;
            if (tt < 0 || tt >= NTH) return;
            constexpr int CPR = BT / 8;
            const int kb = tt / CPR, tq = tt % CPR;       // four k starting at 4*kb, eight columns starting at 8*tq
            const int64_t t = t0 + 8 * tq;
            // a ragged last group of columns is still one 16-byte load where the row pitch covers it (every row but the
            // operand's last, whose padding need not exist): what the padding holds lands in result rows / columns beyond
            // the matrix, which are never stored
            const int exact = t >= T ? 0 : static_cast<int>(T - t < 8 ? T - t : 8);
            const int padded = (exact > 0 && t + 8 <= ld) ? 8 : exact;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int64_t k = k0 + 4 * kb + j;
                r[j] = load8(base, k * ld + t, k < k_end ? (k + 1 < k_rows ? padded : exact) : 0);
            }
        }
    }

    // check-free loads of interior tiles (operand stored along the reduction index): addresses formed once
    const char *pf[NLD];

    __device__ __forceinline__ void fast_begin(const char *base, int64_t ld, int64_t t0, int64_t k0, int tid) {
        static_assert(KC, "the check-free path serves operands stored along the reduction index");
#pragma unroll
        for (int q = 0; q < NLD; ++q) {
            const int idx = tid + 256 * q;
            pf[q] = base + ((t0 + (idx >> 2)) * ld + k0 + 8 * (idx & 3)) * 2;
        }
    }

    __device__ __forceinline__ void fetch_fast() {
#pragma unroll
        for (int q = 0; q < NLD; ++q) {
            r[q] = *reinterpret_cast<const uint4 *>(pf[q]);
            pf[q] += HBK * 2;
        }
    }

    __device__ __forceinline__ void stash(uint16_t (*s)[HBK + HPAD], int tid) const {
        if constexpr (KC) {
#pragma unroll
            for (int q = 0; q < NLD; ++q) {
                const int idx = tid + 256 * q;
                const int row = idx >> 2, kq = idx & 3;
                *reinterpret_cast<uint4 *>(&s[row][chunk_pos(row, kq)]) = r[q];
            }
        } else {
            const int tt = tid - TOFF;
            if (tt < 0 || tt >= NTH) return;
            constexpr int CPR = BT / 8;
            const int kb = tt / CPR, tq = tt % CPR;
            const uint32_t w[4][4] = {{r[0].x, r[0].y, r[0].z, r[0].w}, {r[1].x, r[1].y, r[1].z, r[1].w},
                                      {r[2].x, r[2].y, r[2].z, r[2].w}, {r[3].x, r[3].y, r[3].z, r[3].w}};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                // column 8*tq+e of the four k: the low (e even) or high (e odd) halves of word e/2 of the four rows
                const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
                uint2 v;
                v.x = __builtin_amdgcn_perm(w[1][e >> 1], w[0][e >> 1], sel);
                v.y = __builtin_amdgcn_perm(w[3][e >> 1], w[2][e >> 1], sel);
                const int row = 8 * tq + e;
                *reinterpret_cast<uint2 *>(&s[row][chunk_pos(row, kb >> 1) + 4 * (kb & 1)]) = v;
            }
        }
    }
};

template <bool A_KC, bool B_KC, int BM, int BN>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmArgs g) {
    constexpr int WM = BM / 2, WN = BN / 2;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int LDSROW = HBK + HPAD;
    constexpr int CPITCH = BN + 8;          // row pitch of the staged output tile (16-byte multiple)
    static_assert(BM * CPITCH <= 2 * (BM + BN) * LDSROW, "the staged output tile must fit the operand buffers");
    __shared__ __attribute__((aligned(16))) uint16_t smem[2 * (BM + BN) * LDSROW];
    uint16_t (*As)[BM][LDSROW] = reinterpret_cast<uint16_t (*)[BM][LDSROW]>(smem);
    uint16_t (*Bs)[BN][LDSROW] = reinterpret_cast<uint16_t (*)[BN][LDSROW]>(smem + 2 * BM * LDSROW);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, half = lane >> 5;
    int bx, by, bz;
    if (!tile_coords(g, &bx, &by, &bz)) return;      // uniform over the workgroup
    const int64_t m0 = static_cast<int64_t>(by) * BM;
    const int64_t n0 = static_cast<int64_t>(bx) * BN;
    const int64_t k_begin = static_cast<int64_t>(bz) * g.k_chunk;
    const int64_t k_end = (k_begin + g.k_chunk < g.K) ? k_begin + g.k_chunk : g.K;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    HalfTileLoader<A_KC, BM, 0> la;
    HalfTileLoader<B_KC, BN, A_KC ? 0 : 128> lb;     // when both operands are transposed they split the threads
    la.k_rows = g.K; lb.k_rows = g.K;
    const int64_t nk = (k_end > k_begin) ? (k_end - k_begin + HBK - 1) / HBK : 0;
    if (nk > 0) {
        la.fetch(g.A, g.lda, m0, g.M, k_begin, k_end, tid);
        lb.fetch(g.B, g.ldb, n0, g.N, k_begin, k_end, tid);
        la.stash(As[0], tid);
        lb.stash(Bs[0], tid);
    }
    // uniform over the workgroup: both operands are stored along the reduction index and the tile lies inside
    constexpr bool FAST = A_KC && B_KC;
    const bool interior = FAST && m0 + BM <= g.M && n0 + BN <= g.N;
    const int64_t nk_full = (k_end > k_begin) ? (k_end - k_begin) / HBK : 0;
    if constexpr (FAST) {
        if (interior) {
            la.fast_begin(g.A, g.lda, m0, k_begin + HBK, tid);
            lb.fast_begin(g.B, g.ldb, n0, k_begin + HBK, tid);
        }
    }
    __syncthreads();
    for (int64_t kt = 0; kt < nk; ++kt) {
        const int buf = static_cast<int>(kt & 1);
        const bool more = kt + 1 < nk;
        if (more) {
            bool done = false;
            if constexpr (FAST) {
                if (interior && kt + 1 < nk_full) {
                    la.fetch_fast();
                    lb.fetch_fast();
                    done = true;
                }
            }
            if (!done) {
                la.fetch(g.A, g.lda, m0, g.M, k_begin + (kt + 1) * HBK, k_end, tid);
                lb.fetch(g.B, g.ldb, n0, g.N, k_begin + (kt + 1) * HBK, k_end, tid);
            }
        }
#pragma unroll
        for (int ks = 0; ks < HBK; ks += 16) {
            bf16x8 a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int row = wm * WM + i * 32 + l32;
                a[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(&As[buf][row][chunk_pos(row, ks / 8 + half)]));
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int row = wn * WN + j * 32 + l32;
                b[j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(&Bs[buf][row][chunk_pos(row, ks / 8 + half)]));
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        if (more) {
            la.stash(As[buf ^ 1], tid);
            lb.stash(Bs[buf ^ 1], tid);
        }
        __syncthreads();
    }
    if (!g.c_staged) {
        store_tile<TM, TN>(g, acc, m0 + wm * WM, n0 + wn * WN, l32, half, bz);
        return;
    }
    // bf16 output without a read-modify-write epilogue: the tile is rounded into LDS (the operand buffers are free
    // after the last barrier) and leaves in 16-byte pieces along the rows, instead of 2 bytes per lane.
    uint16_t (*Cs)[CPITCH] = reinterpret_cast<uint16_t (*)[CPITCH]>(smem);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = wn * WN + j * 32 + l32;
            const float bv = (g.bias && n0 + col < g.N) ? g.bias[n0 + col] : 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = wm * WM + i * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
                float v = acc[i][j][r] + bv;
                if (g.relu) v = v > 0.f ? v : 0.f;
                Cs[row][col] = static_cast<uint16_t>(f32_to_bf16_rne(v));
            }
        }
    __syncthreads();
    constexpr int CQ = BN / 8;
    for (int c = tid; c < BM * CQ; c += 256) {
        const int row = c / CQ, cq = c % CQ;
        const int64_t grow = m0 + row, gcol = n0 + 8 * cq;
        if (grow >= g.M || gcol >= g.N) continue;
        uint16_t *dst = reinterpret_cast<uint16_t *>(g.C) + grow * g.ldc + gcol;
        if (gcol + 8 <= g.N) {
            *reinterpret_cast<uint4 *>(dst) = *reinterpret_cast<const uint4 *>(&Cs[row][8 * cq]);
        } else {
            for (int e = 0; gcol + e < g.N; ++e) dst[e] = Cs[row][8 * cq + e];
        }
    }
}

// ---------------------------------------------------------------------------------------------------
// fp32 operands on the bf16 matrix cores.  An fp32 number is the exact sum of three bf16 numbers (its 24 significant
// bits cut into 8 + 8 + 8, with signs), so a product a * b is the sum of nine bf16 products, each exact in fp32.  The
// three smallest (together at most 2^-23 of the product: the size of fp32's own rounding) are dropped, the other six
// are accumulated in fp32 by v_mfma_f32_32x32x16_bf16, smallest first.  Six such instructions cover the k-range of
// eight v_mfma_f32_32x32x2_f32 at about a fifteenth of the cost each.
//
// LDS holds the three pieces of both operand tiles, 32 k per step, in one buffer (the next step's operands wait in
// registers; two workgroups share a compute unit and fill one another's barriers).  An operand stored along the
// reduction index is cut while it is staged and kept in 16-byte units S[piece][k / 8][row] (a lane's eight k are one
// 16-byte read, consecutive lanes read consecutive units; a plane is 32 bytes longer than a power of two so that the
// 8-byte staging stores of 16 consecutive lanes, 2 rows x 4 units x 2 halves, cover 128 consecutive bytes of banks);
// the weight matrix of a plain product is cut once, by split_repack_kernel, into the same units in global memory and
// only copied here; an operand stored across the reduction index (both operands of X^T G) is transposed in registers
// and kept in 8-byte units S[piece][k / 4][row], which makes both the staging stores (32 bytes per thread and piece)
// and the operand reads (two 8-byte reads) run over consecutive LDS addresses.
constexpr int SBK = 32;

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// two fp32 numbers rounded to bf16 (nearest even), the first in the low half: one v_cvt_pk_bf16_f32
__device__ __forceinline__ uint32_t bf16_pair(float x0, float x1) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2{x0, x1}), bf16x2));
}

// x = piece 0 + piece 1 + piece 2 exactly, for two numbers at once; p[i] holds piece i of x0 in its low half and of
// x1 in its high half.  Rounding to nearest bounds the second piece by 2^-8 |x| and the third by 2^-16 |x|; the
// remainders are exact fp32 differences with at most 16 and 8 significant bits.
__device__ __forceinline__ void split3_pair(float x0, float x1, uint32_t (&p)[3]) {
    p[0] = bf16_pair(x0, x1);
    const float r0 = x0 - __uint_as_float(p[0] << 16), r1 = x1 - __uint_as_float(p[0] & 0xffff0000u);
    p[1] = bf16_pair(r0, r1);
    const float s0 = r0 - __uint_as_float(p[1] << 16), s1 = r1 - __uint_as_float(p[1] & 0xffff0000u);
    p[2] = bf16_pair(s0, s1);
}

// 16-byte units of an operand kept along the reduction index: unit (piece, u = k / 8, row)
template <int BT>
struct Units16 {
    static constexpr int PLANE = BT + 2;                    // units per (piece, u) plane
    static constexpr int BYTES = 3 * 4 * PLANE * 16;
    static __device__ __forceinline__ int at(int piece, int u, int row) { return ((piece * 4 + u) * PLANE + row) * 16; }
};

// operand stored along the reduction index, cut while staged: a row's 32 k are eight float4 of eight threads
template <int BT, int NT = 256>
struct SplitRowLoader {
    static constexpr int NLD = BT * SBK / 4 / NT;
    float4 r[NLD];
    const char *pf[NLD];

    __device__ __forceinline__ void fetch(const char *base, int64_t ld, int64_t t0, int64_t T, int64_t k0, int64_t k_end,
                                          int vec, int tid) {
#pragma unroll
        for (int q = 0; q < NLD; ++q) {
            const int idx = tid + NT * q;
            const int row = idx >> 3, kq = idx & 7;
            const int64_t t = t0 + row, k = k0 + 4 * kq;
            const int nv = (t < T) ? static_cast<int>(k_end - k < 4 ? k_end - k : 4) : 0;
            r[q] = load4<false>(base, t * ld + k, nv, vec);
        }
    }

    __device__ __forceinline__ void fast_begin(const char *base, int64_t ld, int64_t t0, int64_t k0, int tid) {
#pragma unroll
        for (int q = 0; q < NLD; ++q) {
            const int idx = tid + NT * q;
            pf[q] = base + ((t0 + (idx >> 3)) * ld + k0 + 4 * (idx & 7)) * 4;
        }
    }

    __device__ __forceinline__ void fetch_fast() {
#pragma unroll
        for (int q = 0; q < NLD; ++q) {
            r[q] = *reinterpret_cast<const float4 *>(pf[q]);
            pf[q] += SBK * 4;
        }
    }

    // check-free loads of one step at a given place (rows t0.., 32 k from k0): no state between steps.  The tile's
    // corner is uniform over the workgroup, a thread adds a 32-bit offset inside the tile (ld < 2^22 elements).
    __device__ __forceinline__ void fetch_at(const char *base, int64_t ld, int64_t t0, int64_t k0, int tid) {
        const char *corner = base + (t0 * ld + k0) * 4;
#pragma unroll
        for (int q = 0; q < NLD; ++q) {
            const int idx = tid + NT * q;
            const uint32_t off = (static_cast<uint32_t>(idx >> 3) * static_cast<uint32_t>(ld) + 4u * (idx & 7)) * 4u;
            r[q] = *reinterpret_cast<const float4 *>(corner + off);
        }
    }

    uint2 pk[NLD][3];               // the pieces of r, ready for LDS

    __device__ __forceinline__ void cut() {
#pragma unroll
        for (int q = 0; q < NLD; ++q) {
            uint32_t lo[3], hi[3];
            split3_pair(r[q].x, r[q].y, lo);
            split3_pair(r[q].z, r[q].w, hi);
#pragma unroll
            for (int p = 0; p < 3; ++p) pk[q][p] = make_uint2(lo[p], hi[p]);
        }
    }

    __device__ __forceinline__ void put(char *s, int tid) const {
#pragma unroll
        for (int q = 0; q < NLD; ++q) {
            const int idx = tid + NT * q;
            const int row = idx >> 3, kq = idx & 7;
#pragma unroll
            for (int p = 0; p < 3; ++p)
                *reinterpret_cast<uint2 *>(s + Units16<BT>::at(p, kq >> 1, row) + 8 * (kq & 1)) = pk[q][p];
        }
    }
};

// second operand already cut into units Wt[piece][k / 8][n] (n padded to whole tiles, k to whole steps): plain copies
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int BT, int NT = 256>
struct SplitPlaneLoader {
    static constexpr int NLD = 3 * 4 * BT / NT;
    u32x4 r[NLD];
    const u32x4 *pf;                // the thread's first unit; its others lie q * stride_q further on
    int64_t stride_q;               // in units

    // ku_total: 16-byte units along k of one piece; n_pad: rows of a plane.  NT consecutive units of the LDS image
    // (piece, u, row) are NT / BT planes of BT rows: thread tid copies row tid % BT of planes tid / BT + q * NT / BT.
    __device__ __forceinline__ void begin(const uint16_t *Wt, int64_t ku_total, int64_t n_pad, int64_t t0, int64_t k0, int tid) {
        static_assert((BT == 128 || BT == 64) && (NT / BT == 2 || NT / BT == 4), "planes per pass: 2 or 4, both divide the 4 units of a piece");
        const int pu = tid / BT, row = tid % BT;
        pf = reinterpret_cast<const u32x4 *>(Wt) + (k0 / 8 + pu) * n_pad + t0 + row;
        stride_q = (NT / BT) * n_pad;
        piece_stride = (ku_total - 4) * n_pad;
    }
    int64_t piece_stride;           // extra distance when q crosses into the next piece

    __device__ __forceinline__ void fetch(int64_t n_pad) {
        constexpr int PPQ = NT / BT;           // planes per pass
#pragma unroll
        for (int q = 0; q < NLD; ++q) r[q] = pf[q * stride_q + ((q * PPQ) / 4) * piece_stride];
        pf += (SBK / 8) * n_pad;
    }

    __device__ __forceinline__ void stash(char *s, int tid) const {
        constexpr int PPQ = NT / BT;
        const int pu0 = tid / BT, row = tid % BT;
#pragma unroll
        for (int q = 0; q < NLD; ++q) {
            const int pu = pu0 + q * PPQ;
            *reinterpret_cast<u32x4 *>(s + Units16<BT>::at(pu >> 2, pu & 3, row)) = r[q];
        }
    }
};

typedef float f32x4 __attribute__((ext_vector_type(4)));

// LDS image of an operand stored across the reduction index (both of X^T G): 8-byte units (piece, k / 4, column), a
// plane of bt columns per (piece, k / 4).  A staging thread holds four neighbouring columns (32 bytes) and stores them
// as two 16-byte halves; eight neighbouring lanes are 32 bytes apart, so every second group of four lanes swaps its
// halves and one store covers all the banks.  col_slot() is where a column ends up.
struct ColUnits8 {
    static constexpr int bytes(int bt) { return 3 * 8 * bt * 8; }
    static __device__ __forceinline__ int col_slot(int col) { return col ^ ((col >> 3) & 2); }
};

// C = A B (or A B^T) with A stored along the reduction index; the second operand comes cut into units (Wt: ku_total
// units along k per piece, n_pad rows).  NW waves: four (2 x 2) or, on a 128 x 128 tile, eight (2 x 4, each a 64 x 32
// part: half the staging and half the accumulators per thread, four waves per SIMD).
template <int BM, int BN, int NW = 4, bool DUAL = false>
__global__ __launch_bounds__(NW * 64, NW / 2) void gemm_split_kernel(GemmArgs g, const uint16_t *Wt, int64_t ku_total, int64_t n_pad) {
    static_assert(NW == 4 || (NW == 8 && BN == 128), "eight waves: 128 columns");
    constexpr int NT = NW * 64;
    constexpr int WM = BM / 2, WN = BN / (NW / 2);
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int A_BYTES = Units16<BM>::BYTES;
    constexpr int B_BYTES = Units16<BN>::BYTES;
    __shared__ __attribute__((aligned(16))) char smem[A_BYTES + B_BYTES];
    char *As = smem, *Bs = smem + A_BYTES;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / (NW / 2), wn = wave % (NW / 2);
    const int l32 = lane & 31, half = lane >> 5;
    int bx, by, bz;
    if (!tile_coords(g, &bx, &by, &bz)) return;      // uniform over the workgroup
    const int64_t m0 = static_cast<int64_t>(by) * BM;
    const int64_t n0 = static_cast<int64_t>(bx) * BN;
    const int64_t k_begin = static_cast<int64_t>(bz) * g.k_chunk;
    const int64_t k_end = (k_begin + g.k_chunk < g.K) ? k_begin + g.k_chunk : g.K;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    SplitRowLoader<BM, NT> la_r;
    SplitPlaneLoader<BN, NT> lb_p;
    const int64_t nk = (k_end > k_begin) ? (k_end - k_begin + SBK - 1) / SBK : 0;
    const int64_t nk_full = (k_end > k_begin) ? (k_end - k_begin) / SBK : 0;
    // uniform over the workgroup: every row of the tile exists and vector loads are allowed
    const bool interior = m0 + BM <= g.M && g.a_vec;
    if (nk > 0) {
        la_r.fetch(g.A, g.lda, m0, g.M, k_begin, DUAL ? g.K1 : k_end, g.a_vec, tid);      // DUAL: one split, k_begin = 0
        lb_p.begin(Wt, ku_total, n_pad, n0, k_begin, tid);
        lb_p.fetch(n_pad);
        la_r.cut();
        la_r.put(As, tid);
        lb_p.stash(Bs, tid);
        if (!DUAL && interior) la_r.fast_begin(g.A, g.lda, m0, k_begin + SBK, tid);
    }
    __syncthreads();
    // the products of one step (32 k) out of LDS; CUT: the first operand of the next step, which waits in registers, is
    // cut into its pieces between the matrix instructions of the second half (about five vector instructions fit
    // behind each matrix instruction's issue; measured: 4 %)
    auto products = [&](auto cut_tag) {
        constexpr bool CUT = decltype(cut_tag)::value;
#pragma unroll
        for (int ks = 0; ks < SBK / 16; ++ks) {
            // nothing of the second half moves into the first: the loads of the next operands get that long to arrive
            if (CUT && ks == SBK / 16 - 1) __builtin_amdgcn_sched_barrier(0);
            bf16x8 a[3][TM], b[3][TN];
#pragma unroll
            for (int p = 0; p < 3; ++p) {
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    const int row = wm * WM + i * 32 + l32;
                    a[p][i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(As + Units16<BM>::at(p, 2 * ks + half, row)));
                }
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int row = wn * WN + j * 32 + l32;
                    b[p][j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(Bs + Units16<BN>::at(p, 2 * ks + half, row)));
                }
            }
            if (CUT && ks == SBK / 16 - 1) la_r.cut();
            // the six piece products, smallest first
#define CG_PIECES(PA_, PB_)                                                                                                  \
    _Pragma("unroll") for (int i = 0; i < TM; ++i) _Pragma("unroll") for (int j = 0; j < TN; ++j)                            \
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[PA_][i], b[PB_][j], acc[i][j], 0, 0, 0);
            CG_PIECES(2, 0) CG_PIECES(0, 2) CG_PIECES(1, 1) CG_PIECES(1, 0) CG_PIECES(0, 1) CG_PIECES(0, 0)
#undef CG_PIECES
            if (CUT && ks == SBK / 16 - 1) {
#pragma unroll
                for (int t = 0; t < 6 * TM * TN; ++t) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);      // one matrix instruction
                    __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);      // vector instructions behind it
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    for (int64_t kt = 0; kt + 1 < nk; ++kt) {
        if constexpr (DUAL) {
            // which of the two first operands this step reads is uniform over the grid; the check-free loads form their
            // addresses from it (no per-thread pointers to carry across the change of operand)
            const int64_t k0 = (kt + 1) * SBK;
            const bool second = k0 >= g.K1p;
            const char *base = second ? g.A2 : g.A;
            const int64_t ld = second ? g.lda2 : g.lda;
            const int64_t kk = second ? k0 - g.K1p : k0, kend = second ? g.K - g.K1p : g.K1;
            if (interior && kk + SBK <= kend) la_r.fetch_at(base, ld, m0, kk, tid);
            else la_r.fetch(base, ld, m0, g.M, kk, kend, g.a_vec, tid);
        } else {
            if (interior && kt + 1 < nk_full) la_r.fetch_fast();
            else la_r.fetch(g.A, g.lda, m0, g.M, k_begin + (kt + 1) * SBK, k_end, g.a_vec, tid);
        }
        lb_p.fetch(n_pad);
        products(std::true_type{});
        __syncthreads();            // every wave has read this step's operands
        la_r.put(As, tid);
        lb_p.stash(Bs, tid);
        __syncthreads();
    }
    if (nk > 0) products(std::false_type{});
    if constexpr (TM == 2 && (TN == 2 || TN == 1)) {
        static_assert(NW * STAGE_BYTES_T<TN> <= A_BYTES + B_BYTES, "the staged output must fit the operand buffers");
        __syncthreads();                    // every wave is done with the operands
        store_tile_staged<TN>(g, acc, reinterpret_cast<float *>(smem + wave * STAGE_BYTES_T<TN>), m0 + wm * WM, n0 + wn * WN, lane, bz);
    } else {
        store_tile<TM, TN>(g, acc, m0 + wm * WM, n0 + wn * WN, l32, half, bz);
    }
}

// The weight gradient with eight waves on a 128 x BN tile (BN = 128: 2 x 4 waves, each a 64 x 32 part; BN = 64: 4 x 2,
// each 32 x 32): half the staging and at most half the accumulators per thread of the four-wave form, so that four
// waves share a SIMD and one wave's cutting and LDS traffic run beside another's matrix instructions.  Waves 0-3 stage
// the first operand's tile, waves 4-7 the second's; LDS image as in gemm_split_kernel<true, ...>: 8-byte units
// (piece, k / 4, column), columns placed by ColUnits8::col_slot.
struct SplitColLoader {
    f32x4 r[4];                     // one block of 4 k x 4 columns per thread
    const f32x4 *pf;
    const char *base;
    int64_t ld, t0, T;
    char *s;
    int bt, kb, tq;                 // tile width; the thread's k-block and column group
    bool idle;                      // a 64-column second tile leaves half of its waves without work
    uint2 pk[4][3];                 // [column][piece], four k each

    __device__ __forceinline__ void init(const GemmArgs &g, int64_t m0, int64_t n0, int bm, int bn, char *As, char *Bs, int tid) {
        const bool second = __builtin_amdgcn_readfirstlane(tid >> 8) != 0;        // uniform over the wave
        base = second ? g.B : g.A;
        ld = second ? g.ldb : g.lda;
        t0 = second ? n0 : m0;
        T = second ? g.N : g.M;
        s = second ? Bs : As;
        bt = second ? bn : bm;
        const int tt = tid & 255, cpr = bt / 4;
        kb = tt / cpr; tq = tt % cpr;
        idle = kb >= 8;
    }

    __device__ __forceinline__ void fetch(int64_t k0, int64_t k_end, int vec) {
        if (idle) return;
        const int64_t t = t0 + 4 * tq;
        const int ncol = static_cast<int>(T - t < 4 ? T - t : 4);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t k = k0 + 4 * kb + j;
            const float4 v = load4<false>(base, k * ld + t, k < k_end ? ncol : 0, vec);
            r[j] = f32x4{v.x, v.y, v.z, v.w};
        }
    }

    __device__ __forceinline__ void fast_begin(int64_t k0) {
        pf = reinterpret_cast<const f32x4 *>(base + ((k0 + 4 * kb) * ld + t0 + 4 * tq) * 4);
    }

    // the check-free path runs only when rows are whole 16-byte vectors
    __device__ __forceinline__ void fetch_fast() {
        if (idle) return;
        const int64_t ld4 = ld / 4;
#pragma unroll
        for (int j = 0; j < 4; ++j) r[j] = pf[j * ld4];
        pf += SBK * ld4;
    }

    __device__ __forceinline__ void cut() {
        if (idle) return;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            uint32_t lo[3], hi[3];
            split3_pair(r[0][c], r[1][c], lo);
            split3_pair(r[2][c], r[3][c], hi);
#pragma unroll
            for (int p = 0; p < 3; ++p) pk[c][p] = make_uint2(lo[p], hi[p]);
        }
    }

    __device__ __forceinline__ void put() const {
        if (idle) return;
        const int sw = ((tq >> 2) & 1) * 16;       // see ColUnits8
#pragma unroll
        for (int p = 0; p < 3; ++p) {
            char *dst = s + (((p * 8 + kb) * bt) + 4 * tq) * 8;
            *reinterpret_cast<uint4 *>(dst + sw) = make_uint4(pk[0][p].x, pk[0][p].y, pk[1][p].x, pk[1][p].y);
            *reinterpret_cast<uint4 *>(dst + 16 - sw) = make_uint4(pk[2][p].x, pk[2][p].y, pk[3][p].x, pk[3][p].y);
        }
    }
};

template <int BN>
// (second launch bound: waves per SIMD; two workgroups of eight waves per compute unit need four)
__global__ __launch_bounds__(512, BN == 128 ? 4 : 2) void gemm_split_trans_kernel(GemmArgs g) {
    static_assert(BN == 128 || BN == 64, "tile widths");
    constexpr int BM = 128;
    constexpr int WAVES_N = BN / 32, WAVES_M = 8 / WAVES_N;     // every wave one 32-column strip
    constexpr int WM = BM / WAVES_M, WN = 32, TM = WM / 32;
    constexpr int A_BYTES = ColUnits8::bytes(BM), B_BYTES = ColUnits8::bytes(BN);
    __shared__ __attribute__((aligned(16))) char smem[A_BYTES + B_BYTES];
    char *As = smem, *Bs = smem + A_BYTES;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int l32 = lane & 31, half = lane >> 5;
    int bx, by, bz;
    if (!tile_coords(g, &bx, &by, &bz)) return;      // uniform over the workgroup
    const int64_t m0 = static_cast<int64_t>(by) * BM;
    const int64_t n0 = static_cast<int64_t>(bx) * BN;
    const int64_t k_begin = static_cast<int64_t>(bz) * g.k_chunk;
    const int64_t k_end = (k_begin + g.k_chunk < g.K) ? k_begin + g.k_chunk : g.K;

    floatx16 acc[TM][1];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][0][r] = 0.f;

    SplitColLoader lc;
    const int64_t nk = (k_end > k_begin) ? (k_end - k_begin + SBK - 1) / SBK : 0;
    const int64_t nk_full = (k_end > k_begin) ? (k_end - k_begin) / SBK : 0;
    // uniform over the workgroup: every row / column of the tile exists and vector loads are allowed
    const bool interior = m0 + BM <= g.M && n0 + BN <= g.N && g.a_vec && g.b_vec;
    const int both_vec = g.a_vec && g.b_vec;
    lc.init(g, m0, n0, BM, BN, As, Bs, tid);
    if (nk > 0) {
        lc.fetch(k_begin, k_end, both_vec);
        lc.cut();
        lc.put();
        if (interior) lc.fast_begin(k_begin + SBK);
    }
    __syncthreads();
    const int slot_b = ColUnits8::col_slot(wn * WN + l32);
    auto products = [&]() {
#pragma unroll
        for (int ks = 0; ks < SBK / 16; ++ks) {
            bf16x8 a[3][TM], b[3];
#pragma unroll
            for (int p = 0; p < 3; ++p) {
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    const int slot = ColUnits8::col_slot(wm * WM + i * 32 + l32);
                    const uint2 v0 = *reinterpret_cast<const uint2 *>(As + ((p * 8 + 4 * ks + 2 * half) * BM + slot) * 8);
                    const uint2 v1 = *reinterpret_cast<const uint2 *>(As + ((p * 8 + 4 * ks + 2 * half + 1) * BM + slot) * 8);
                    a[p][i] = __builtin_bit_cast(bf16x8, make_uint4(v0.x, v0.y, v1.x, v1.y));
                }
                const uint2 w0 = *reinterpret_cast<const uint2 *>(Bs + ((p * 8 + 4 * ks + 2 * half) * BN + slot_b) * 8);
                const uint2 w1 = *reinterpret_cast<const uint2 *>(Bs + ((p * 8 + 4 * ks + 2 * half + 1) * BN + slot_b) * 8);
                b[p] = __builtin_bit_cast(bf16x8, make_uint4(w0.x, w0.y, w1.x, w1.y));
            }
            // the six piece products, smallest first
#define CG_PIECES_T(PA_, PB_)                                                                                                 \
    _Pragma("unroll") for (int i = 0; i < TM; ++i)                                                                           \
        acc[i][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[PA_][i], b[PB_], acc[i][0], 0, 0, 0);
            CG_PIECES_T(2, 0) CG_PIECES_T(0, 2) CG_PIECES_T(1, 1) CG_PIECES_T(1, 0) CG_PIECES_T(0, 1) CG_PIECES_T(0, 0)
#undef CG_PIECES_T
        }
    };
    for (int64_t kt = 0; kt + 1 < nk; ++kt) {
        if (interior && kt + 1 < nk_full) lc.fetch_fast();
        else lc.fetch(k_begin + (kt + 1) * SBK, k_end, both_vec);
        products();
        __syncthreads();            // every wave has read this step's operands
        lc.cut();
        lc.put();
        __syncthreads();
    }
    if (nk > 0) products();
    store_tile<TM, 1>(g, acc, m0 + wm * WM, n0 + wn * WN, l32, half, bz);
}

// Cuts the (small) second operand of a plain product into bf16 pieces laid out in 16-byte units
// Wt[piece][k / 8][n][k % 8], n_pad rows, ku_total units along k, zero beyond N and K.  kc: the source is [n][k]
// (pitch ldw), else [k][n].
// A second source W2 (K2 rows, or columns when kc) follows from k = K1p on.
__global__ __launch_bounds__(256) void split_repack_kernel(const float *W, int64_t ldw, int kc, int64_t K, int64_t N,
                                                           uint16_t *Wt, int64_t n_pad, int64_t ku_total,
                                                           const float *W2 = nullptr, int64_t ldw2 = 0, int64_t K1p = 0,
                                                           int64_t K2 = 0) {
    const int64_t t = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    const int64_t plane = ku_total * n_pad * 8;
    if (t >= plane) return;
    const int64_t ku = t / (n_pad * 8), n = (t / 8) % n_pad, k = 8 * ku + (t % 8);
    float x = (n < N && k < K) ? (kc ? W[n * ldw + k] : W[k * ldw + n]) : 0.f;
    if (W2 && k >= K1p) {
        const int64_t k2 = k - K1p;
        x = (n < N && k2 < K2) ? (kc ? W2[n * ldw2 + k2] : W2[k2 * ldw2 + n]) : 0.f;
    }
    uint32_t p[3];
    split3_pair(x, 0.f, p);
    Wt[t] = static_cast<uint16_t>(p[0]);
    Wt[plane + t] = static_cast<uint16_t>(p[1]);
    Wt[2 * plane + t] = static_cast<uint16_t>(p[2]);
}

// Lays the (small) second operand of a product out as Wt[n][k], k contiguous, rows padded to 16 bytes, for the
// bf16 kernel.  kc: the source already is [n][k] (pitch ldw), else it is [k][n].
__global__ __launch_bounds__(256) void repack_bf16_kernel(const uint16_t *W, int64_t ldw, int kc, int64_t K, int64_t N,
                                                          uint16_t *Wt, int64_t ldt) {
    const int64_t t = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (t >= N * ldt) return;
    const int64_t n = t / ldt, k = t % ldt;
    Wt[t] = k < K ? (kc ? W[n * ldw + k] : W[k * ldw + n]) : static_cast<uint16_t>(0);
}

// Sums the split partials and applies the epilogue.  A workgroup covers 32 consecutive output elements with 8
// groups of threads; group y adds the partials z = y, y+8, ... in that order, then the 8 group sums are added
// in group order: a fixed summation order, whatever the launch geometry.
__global__ __launch_bounds__(256) void gemm_reduce_kernel(GemmArgs g, int S) {
    __shared__ float red[8][32];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int64_t total = g.M * g.N;
    const int64_t t = static_cast<int64_t>(blockIdx.x) * 32 + tx;
    float v = 0.f;
    if (t < total)
        for (int z = ty; z < S; z += 8) v += g.part[static_cast<int64_t>(z) * total + t];
    red[ty][tx] = v;
    __syncthreads();
    if (ty != 0 || t >= total) return;
    v = 0.f;
    for (int y = 0; y < 8; ++y) v += red[y][tx];
    const int64_t row = t / g.N, col = t % g.N;
    if (g.accumulate) {
        v += g.out_bf16 ? __uint_as_float(static_cast<uint32_t>(reinterpret_cast<const uint16_t *>(g.C)[row * g.ldc + col]) << 16)
                        : reinterpret_cast<const float *>(g.C)[row * g.ldc + col];
    }
    if (g.bias) v += g.bias[col];
    if (g.relu) v = v > 0.f ? v : 0.f;
    if (g.mask) {
        const float mv = g.mask_bf16 ? __uint_as_float(static_cast<uint32_t>(reinterpret_cast<const uint16_t *>(g.mask)[row * g.ldm + col]) << 16)
                                     : reinterpret_cast<const float *>(g.mask)[row * g.ldm + col];
        if (!(mv > 0.f)) v = 0.f;
    }
    if (g.rscale) v *= g.rscale[row];
    if (g.out_bf16) reinterpret_cast<uint16_t *>(g.C)[row * g.ldc + col] = static_cast<uint16_t>(f32_to_bf16_rne(v));
    else reinterpret_cast<float *>(g.C)[row * g.ldc + col] = v;
}

static int choose_split(int trans_a, int64_t M, int64_t N, int64_t K, int bm, int bn, int bk) {
    if (!trans_a) return 1;
    const int64_t tiles = ((M + bm - 1) / bm) * ((N + bn - 1) / bn);
    int64_t s = 1536 / (tiles > 0 ? tiles : 1);
    const int64_t max_by_k = K / (bk * 16) > 0 ? K / (bk * 16) : 1;   // at least 16 k-steps per split
    if (s > max_by_k) s = max_by_k;
    if (s > 1024) s = 1024;
    if (s < 1) s = 1;
    return static_cast<int>(s);
}

static void tile_for(int64_t N, int *bm, int *bn) {
    *bm = 128;
    *bn = (N <= 64) ? 64 : 128;
}

static size_t transposed_b_bytes(int64_t N, int64_t K) {
    return align_up(static_cast<size_t>(N) * ((K + 7) / 8 * 8) * sizeof(uint16_t), 256);
}

// the three bf16 planes of an fp32 weight matrix: rows padded to whole tiles, k to whole steps
static int64_t split_rows(int64_t N) { return (N + 127) / 128 * 128; }
static int64_t split_ld(int64_t K) { return (K + SBK - 1) / SBK * SBK; }
static size_t split_b_bytes(int64_t N, int64_t K) {
    return align_up(static_cast<size_t>(3) * split_rows(N) * split_ld(K) * sizeof(uint16_t), 256);
}

size_t gemm_ws_bytes(int trans_a, int64_t M, int64_t N, int64_t K) {
    int bm, bn;
    tile_for(N, &bm, &bn);
    // the larger split of the two kernels (they step through K in 16s and 32s)
    const int s = std::max(choose_split(trans_a, M, N, K, bm, bn, BK), choose_split(trans_a, M, N, K, bm, bn, HBK));
    size_t b = s > 1 ? align_up(static_cast<size_t>(s) * M * N * sizeof(float), 256) : 0;
    // room to lay a weight matrix out for the bf16 kernel (bf16 operands) or as its three planes (fp32 operands)
    if (!trans_a) b = std::max(b, std::max(transposed_b_bytes(N, K), split_b_bytes(N, K)));
    return b;
}

size_t gemm_dual_ws_bytes(int64_t N, int64_t K1, int64_t K2) { return split_b_bytes(N, split_ld(K1) + K2); }

// AUTO: smaller products stay on the fp32 instruction, and so do weight gradients at most 64 columns wide (half of
// the threads that stage their operands would idle; measured slower)
constexpr int64_t SPLIT_MIN_MACS = int64_t(1) << 28;

// tiles 64 columns wide keep four waves; 128-column tiles run eight (both forms of the product)
static void launch_split_tiles(bool trans, const GemmArgs &g, int bn, dim3 grid, const uint16_t *Wt, int64_t ku_total,
                               int64_t n_pad, hipStream_t st) {
    if (trans) {
        if (bn == 64) hipLaunchKernelGGL(gemm_split_trans_kernel<64>, grid, dim3(512), 0, st, g);
        else hipLaunchKernelGGL(gemm_split_trans_kernel<128>, grid, dim3(512), 0, st, g);
    } else {
        if (bn == 64) hipLaunchKernelGGL((gemm_split_kernel<128, 64>), grid, dim3(256), 0, st, g, Wt, ku_total, n_pad);
        else hipLaunchKernelGGL((gemm_split_kernel<128, 128, 8>), grid, dim3(512), 0, st, g, Wt, ku_total, n_pad);
    }
}

template <bool BF16, bool A_KC, bool B_KC>
static void launch_tiles(const GemmArgs &g, int bn, dim3 grid, hipStream_t st) {
    if (bn == 64) hipLaunchKernelGGL((gemm_kernel<BF16, A_KC, B_KC, 128, 64>), grid, dim3(256), 0, st, g);
    else hipLaunchKernelGGL((gemm_kernel<BF16, A_KC, B_KC, 128, 128>), grid, dim3(256), 0, st, g);
}

template <bool A_KC, bool B_KC>
static void launch_bf16_tiles(const GemmArgs &g, int bn, dim3 grid, hipStream_t st) {
    if (bn == 64) hipLaunchKernelGGL((gemm_bf16_kernel<A_KC, B_KC, 128, 64>), grid, dim3(256), 0, st, g);
    else hipLaunchKernelGGL((gemm_bf16_kernel<A_KC, B_KC, 128, 128>), grid, dim3(256), 0, st, g);
}

int launch_gemm(int trans_a, int trans_b, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda,
                const void *B, int64_t ldb, void *C, int64_t ldc, int dtype, int out_f32, int accumulate,
                const float *bias, int relu, const void *relu_mask, int64_t ldm, void *ws, size_t ws_bytes,
                hipStream_t stream, const float *row_scale, int f32_product) {
    if (dtype != CAPGNN_F32 && dtype != CAPGNN_BF16) CG_FAIL(CAPGNN_EINVAL, "gemm: unknown dtype %d", dtype);
    if (f32_product != CAPGNN_F32_PRODUCT_AUTO && f32_product != CAPGNN_F32_PRODUCT_NATIVE && f32_product != CAPGNN_F32_PRODUCT_SPLIT)
        CG_FAIL(CAPGNN_EINVAL, "gemm: unknown form of the fp32 product %d", f32_product);
    if (M < 0 || N < 0 || K < 0) CG_FAIL(CAPGNN_EINVAL, "gemm: negative size");
    if (M == 0 || N == 0) return CAPGNN_OK;
    if (!A || !B || !C) CG_FAIL(CAPGNN_EINVAL, "gemm: NULL operand");
    if (lda < (trans_a ? M : K) || ldb < (trans_b ? K : N) || ldc < N || (relu_mask && ldm < N))
        CG_FAIL(CAPGNN_EINVAL, "gemm: leading dimension too small");
    if (M >= (int64_t(1) << 31) * 64 || N > (1 << 22)) CG_FAIL(CAPGNN_EINVAL, "gemm: size out of range");
    const int es = elem_bytes(dtype);
    int bm, bn;
    tile_for(N, &bm, &bn);
    // bf16 operands whose rows start on 16-byte boundaries run on the bf16 matrix cores; the second operand of a
    // product with a plain first operand is a weight matrix, small enough to be repacked into the workspace
    const bool repack_b = dtype == CAPGNN_BF16 && !trans_a && ws && ws_bytes >= transposed_b_bytes(N, K);
    const bool half_path = dtype == CAPGNN_BF16 && aligned16(A) && (lda * 2) % 16 == 0 &&
                           (repack_b || (aligned16(B) && (ldb * 2) % 16 == 0));
    // fp32 operands as three bf16 pieces each (see gemm_split_kernel)
    const int mode = f32_product;
    const bool split_path = dtype == CAPGNN_F32 && mode != CAPGNN_F32_PRODUCT_NATIVE && !(trans_a && trans_b) &&
                            (mode == CAPGNN_F32_PRODUCT_SPLIT ||
                             (M * N >= SPLIT_MIN_MACS / (K > 0 ? K : 1) && !(trans_a && N <= 64))) &&
                            (trans_a || (ws && ws_bytes >= split_b_bytes(N, K)));
    const int bk = (half_path || split_path) ? HBK : BK;
    static_assert(SBK == HBK, "the two bf16 kernels step through K alike");
    const int S = choose_split(trans_a, M, N, K, bm, bn, bk);
    GemmArgs g;
    g.M = M; g.N = N; g.K = K;
    g.A = static_cast<const char *>(A); g.lda = lda;
    g.B = static_cast<const char *>(B); g.ldb = ldb;
    g.C = static_cast<char *>(C); g.ldc = ldc;
    g.part = nullptr;
    g.k_chunk = K > 0 ? K : 1;
    const size_t va = 4 * es;   // bytes of one 4-element vector
    g.a_vec = (reinterpret_cast<uintptr_t>(A) % va == 0) && ((lda * es) % va == 0);
    g.b_vec = (reinterpret_cast<uintptr_t>(B) % va == 0) && ((ldb * es) % va == 0);
    g.out_bf16 = (dtype == CAPGNN_BF16 && !out_f32);
    g.accumulate = accumulate; g.relu = relu; g.bias = bias;
    g.mask = static_cast<const char *>(relu_mask); g.ldm = ldm; g.mask_bf16 = (dtype == CAPGNN_BF16);
    g.rscale = row_scale;
    g.A2 = nullptr; g.lda2 = 0; g.K1 = 0; g.K1p = 0;
    if (S > 1) {
        const size_t need = static_cast<size_t>(S) * M * N * sizeof(float);
        if (!ws || ws_bytes < need) CG_FAIL(CAPGNN_ENOMEM, "gemm: workspace of %zu bytes needed, %zu given", need, ws_bytes);
        g.part = static_cast<float *>(ws);
        const int64_t steps = (K + bk - 1) / bk;
        g.k_chunk = (steps + S - 1) / S * bk;
    }
    const int64_t gy = (M + bm - 1) / bm, gx = (N + bn - 1) / bn;
    const int64_t n_wg = S > 1 ? NUM_XCD * ((S + NUM_XCD - 1) / NUM_XCD) * gx * gy : NUM_XCD * ((gy + NUM_XCD - 1) / NUM_XCD) * gx;
    if (n_wg >= (int64_t(1) << 31) || gx >= (int64_t(1) << 24) || gy >= (int64_t(1) << 30))
        CG_FAIL(CAPGNN_EINVAL, "gemm: %lld x %lld tiles exceed the grid", (long long)gy, (long long)gx);
    g.gx = static_cast<int>(gx); g.gy = static_cast<int>(gy); g.S = S;
    g.c_staged = half_path && g.out_bf16 && !g.part && !g.mask && !g.accumulate && !g.rscale && aligned16(C) && (ldc * 2) % 16 == 0;
    dim3 grid(static_cast<unsigned>(n_wg), 1, 1);
    bool akc = !trans_a, bkc = trans_b != 0;
    if (split_path) {
        if (trans_a) {
            launch_split_tiles(true, g, bn, grid, nullptr, 0, 0, stream);
        } else {
            const int64_t n_pad = split_rows(N), ku_total = split_ld(K) / 8;
            hipLaunchKernelGGL(split_repack_kernel, dim3(static_cast<unsigned>((ku_total * n_pad * 8 + 255) / 256)), dim3(256), 0,
                               stream, static_cast<const float *>(B), ldb, bkc ? 1 : 0, K, N, static_cast<uint16_t *>(ws), n_pad,
                               ku_total);
            launch_split_tiles(false, g, bn, grid, static_cast<const uint16_t *>(ws), ku_total, n_pad, stream);
        }
    } else if (half_path) {
        if (repack_b) {
            const int64_t ldt = (K + 7) / 8 * 8;
            hipLaunchKernelGGL(repack_bf16_kernel, dim3(static_cast<unsigned>((N * ldt + 255) / 256)), dim3(256), 0, stream,
                               static_cast<const uint16_t *>(B), ldb, bkc ? 1 : 0, K, N, static_cast<uint16_t *>(ws), ldt);
            g.B = static_cast<const char *>(ws); g.ldb = ldt;
            bkc = true;
        }
        if (akc && bkc) launch_bf16_tiles<true, true>(g, bn, grid, stream);
        else if (akc) launch_bf16_tiles<true, false>(g, bn, grid, stream);
        else if (bkc) launch_bf16_tiles<false, true>(g, bn, grid, stream);
        else launch_bf16_tiles<false, false>(g, bn, grid, stream);
    } else {
        const bool bf = dtype == CAPGNN_BF16;
#define CG_GEMM_CASE(BF, AK, BKC_) if (bf == BF && akc == AK && bkc == BKC_) launch_tiles<BF, AK, BKC_>(g, bn, grid, stream);
        CG_GEMM_CASE(false, true, false) CG_GEMM_CASE(false, true, true)
        CG_GEMM_CASE(false, false, false) CG_GEMM_CASE(false, false, true)
        CG_GEMM_CASE(true, true, false) CG_GEMM_CASE(true, true, true)
        CG_GEMM_CASE(true, false, false) CG_GEMM_CASE(true, false, true)
#undef CG_GEMM_CASE
    }
    CG_HIP(hipGetLastError());
    if (S > 1) {
        const int64_t total = M * N;
        hipLaunchKernelGGL(gemm_reduce_kernel, dim3(static_cast<unsigned>((total + 31) / 32)), dim3(256), 0, stream, g, S);
        CG_HIP(hipGetLastError());
    }
    return CAPGNN_OK;
}

// C = A W + A2 W2 (+ bias, ReLU): the two products of a GraphSAGE layer (neighbour term and self term) into one result.
// fp32 operands in the three-piece form run as ONE launch whose reduction walks A's columns and then A2's, so C is
// written once and never read back; every other case is the two launches it replaces (A2 W2 first, then A W accumulated
// on top with the epilogue).  Plain operands only: A [M x K1], A2 [M x K2], W [K1 x N], W2 [K2 x N], row-major.
int launch_gemm_dual(int64_t M, int64_t N, int64_t K1, const void *A, int64_t lda, const void *W, int64_t ldw, int64_t K2,
                     const void *A2, int64_t lda2, const void *W2, int64_t ldw2, void *C, int64_t ldc, int dtype, int out_f32,
                     const float *bias, int relu, void *ws, size_t ws_bytes, hipStream_t stream, int f32_product) {
    if (f32_product != CAPGNN_F32_PRODUCT_AUTO && f32_product != CAPGNN_F32_PRODUCT_NATIVE && f32_product != CAPGNN_F32_PRODUCT_SPLIT)
        CG_FAIL(CAPGNN_EINVAL, "gemm: unknown form of the fp32 product %d", f32_product);
    const int64_t K1p = split_ld(K1 > 0 ? K1 : 0), K = K1p + K2;
    const bool one_launch = dtype == CAPGNN_F32 && f32_product != CAPGNN_F32_PRODUCT_NATIVE && M > 0 && N > 0 && K1 > 0 && K2 > 0 &&
                            A && A2 && W && W2 && C && lda >= K1 && lda2 >= K2 && ldw >= N && ldw2 >= N && ldc >= N &&
                            N <= (1 << 22) && M < (int64_t(1) << 31) * 64 && lda < (1 << 22) && lda2 < (1 << 22) &&
                            (f32_product == CAPGNN_F32_PRODUCT_SPLIT || M * N >= SPLIT_MIN_MACS / (K1 + K2)) &&
                            ws && ws_bytes >= split_b_bytes(N, K);
    if (!one_launch) {
        CG_TRY(launch_gemm(0, 0, M, N, K2, A2, lda2, W2, ldw2, C, ldc, dtype, out_f32, 0, nullptr, 0, nullptr, 0, ws, ws_bytes,
                           stream, nullptr, f32_product));
        return launch_gemm(0, 0, M, N, K1, A, lda, W, ldw, C, ldc, dtype, out_f32, 1, bias, relu, nullptr, 0, ws, ws_bytes,
                           stream, nullptr, f32_product);
    }
    int bm, bn;
    tile_for(N, &bm, &bn);
    GemmArgs g;
    g.M = M; g.N = N; g.K = K;
    g.A = static_cast<const char *>(A); g.lda = lda;
    g.B = static_cast<const char *>(W); g.ldb = ldw;
    g.C = static_cast<char *>(C); g.ldc = ldc;
    g.part = nullptr;
    g.k_chunk = K;
    g.a_vec = (reinterpret_cast<uintptr_t>(A) % 16 == 0) && ((lda * 4) % 16 == 0) && (reinterpret_cast<uintptr_t>(A2) % 16 == 0) &&
              ((lda2 * 4) % 16 == 0);
    g.b_vec = 0;
    g.out_bf16 = 0; g.accumulate = 0; g.relu = relu; g.bias = bias;
    g.mask = nullptr; g.ldm = 0; g.mask_bf16 = 0;
    g.rscale = nullptr;
    g.A2 = static_cast<const char *>(A2); g.lda2 = lda2; g.K1 = K1; g.K1p = K1p;
    const int64_t gy = (M + bm - 1) / bm, gx = (N + bn - 1) / bn;
    const int64_t n_wg = NUM_XCD * ((gy + NUM_XCD - 1) / NUM_XCD) * gx;
    if (n_wg >= (int64_t(1) << 31) || gx >= (int64_t(1) << 24) || gy >= (int64_t(1) << 30))
        CG_FAIL(CAPGNN_EINVAL, "gemm: %lld x %lld tiles exceed the grid", (long long)gy, (long long)gx);
    g.gx = static_cast<int>(gx); g.gy = static_cast<int>(gy); g.S = 1;
    g.c_staged = 0;
    const int64_t n_pad = split_rows(N), ku_total = split_ld(K) / 8;
    hipLaunchKernelGGL(split_repack_kernel, dim3(static_cast<unsigned>((ku_total * n_pad * 8 + 255) / 256)), dim3(256), 0, stream,
                       static_cast<const float *>(W), ldw, 0, K1, N, static_cast<uint16_t *>(ws), n_pad, ku_total,
                       static_cast<const float *>(W2), ldw2, K1p, K2);
    dim3 grid(static_cast<unsigned>(n_wg), 1, 1);
    if (bn == 64)
        hipLaunchKernelGGL((gemm_split_kernel<128, 64, 4, true>), grid, dim3(256), 0, stream, g, static_cast<const uint16_t *>(ws),
                           ku_total, n_pad);
    else
        hipLaunchKernelGGL((gemm_split_kernel<128, 128, 8, true>), grid, dim3(512), 0, stream, g, static_cast<const uint16_t *>(ws),
                           ku_total, n_pad);
    CG_HIP(hipGetLastError());
    return CAPGNN_OK;
}

// Register-resident matrix-instruction loop: what the matrix cores deliver on this chip when nothing else is in
// the way (four independent 32x32 accumulator tiles per wave, operands never reloaded).  The utilisation figures
// of the product kernels can be read against it as well as against the data-sheet peak.
template <bool BF16>
__global__ __launch_bounds__(256) void mfma_peak_kernel(int iters, float *out) {
    floatx16 acc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
    const float a = 1.f + 1e-3f * threadIdx.x, b = 1.f - 1e-3f * threadIdx.x;
    bf16x8 ha, hb;
#pragma unroll
    for (int j = 0; j < 8; ++j) { ha[j] = static_cast<__bf16>(a); hb[j] = static_cast<__bf16>(b); }
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            if constexpr (BF16) acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ha, hb, acc[t], 0, 0, 0);
            else acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[t], 0, 0, 0);
        }
    }
    float s = 0.f;
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[t][r];
    out[static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x] = s;     // keeps the loop alive
}

}  // namespace capgnn

using namespace capgnn;

extern "C" int capgnn_mfma_peak(int dtype, int workgroups, int iters, float *out, double *flop, void *stream) {
    if ((dtype != CAPGNN_F32 && dtype != CAPGNN_BF16) || workgroups <= 0 || iters <= 0 || !out || !flop)
        CG_FAIL(CAPGNN_EINVAL, "mfma_peak: bad argument");
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dtype == CAPGNN_BF16) hipLaunchKernelGGL(mfma_peak_kernel<true>, dim3(workgroups), dim3(256), 0, st, iters, out);
    else hipLaunchKernelGGL(mfma_peak_kernel<false>, dim3(workgroups), dim3(256), 0, st, iters, out);
    CG_HIP(hipGetLastError());
    const double per_instr = dtype == CAPGNN_BF16 ? 2.0 * 32 * 32 * 16 : 2.0 * 32 * 32 * 2;
    *flop = per_instr * 4.0 * iters * 4.0 * workgroups;     // 4 tiles per wave, 4 waves per workgroup
    return CAPGNN_OK;
}

extern "C" size_t capgnn_gemm_workspace_bytes(int trans_a, int64_t M, int64_t N, int64_t K) {
    return gemm_ws_bytes(trans_a, M, N, K);
}

extern "C" int capgnn_gemm(int trans_a, int trans_b, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda,
                           const void *B, int64_t ldb, void *C, int64_t ldc, int dtype, int out_f32, int accumulate,
                           const float *bias, int relu, const void *relu_mask, int64_t ldm, int f32_product, void *ws,
                           size_t ws_bytes, void *stream) {
    return launch_gemm(trans_a, trans_b, M, N, K, A, lda, B, ldb, C, ldc, dtype, out_f32, accumulate, bias, relu,
                       relu_mask, ldm, ws, ws_bytes, static_cast<hipStream_t>(stream), nullptr, f32_product);
}
