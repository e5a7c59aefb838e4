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
                if (g.out_bf16) reinterpret_cast<uint16_t *>(g.C)[row * g.ldc + col] = static_cast<uint16_t>(f32_to_bf16_rne(v));
                else reinterpret_cast<float *>(g.C)[row * g.ldc + col] = v;
            }
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
    __shared__ __attribute__((aligned(16))) float As[2][BK][BM + PAD];
    __shared__ __attribute__((aligned(16))) float Bs[2][BK][BN + PAD];

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

    store_tile<TM, TN>(g, acc, m0 + wm * WM, n0 + wn * WN, l32, half, bz);
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
            const int ncol = static_cast<int>(T - t < 8 ? T - t : 8);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int64_t k = k0 + 4 * kb + j;
                r[j] = load8(base, k * ld + t, k < k_end ? ncol : 0);
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
    if (g.out_bf16) reinterpret_cast<uint16_t *>(g.C)[row * g.ldc + col] = static_cast<uint16_t>(f32_to_bf16_rne(v));
    else reinterpret_cast<float *>(g.C)[row * g.ldc + col] = v;
}

static int choose_split(int trans_a, int64_t M, int64_t N, int64_t K, int bm, int bn, int bk) {
    if (!trans_a) return 1;
    const int64_t tiles = ((M + bm - 1) / bm) * ((N + bn - 1) / bn);
    int64_t s = 1536 / (tiles > 0 ? tiles : 1);
    const int64_t max_by_k = K / (bk * 16) > 0 ? K / (bk * 16) : 1;   // at least 16 k-steps per split
    if (s > max_by_k) s = max_by_k;
    if (s > 512) s = 512;
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

size_t gemm_ws_bytes(int trans_a, int64_t M, int64_t N, int64_t K) {
    int bm, bn;
    tile_for(N, &bm, &bn);
    // the larger split of the two kernels (they step through K in 16s and 32s)
    const int s = std::max(choose_split(trans_a, M, N, K, bm, bn, BK), choose_split(trans_a, M, N, K, bm, bn, HBK));
    size_t b = s > 1 ? align_up(static_cast<size_t>(s) * M * N * sizeof(float), 256) : 0;
    if (!trans_a) b = std::max(b, transposed_b_bytes(N, K));    // room to lay a bf16 weight out for the bf16 kernel
    return b;
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
                hipStream_t stream) {
    if (dtype != CAPGNN_F32 && dtype != CAPGNN_BF16) CG_FAIL(CAPGNN_EINVAL, "gemm: unknown dtype %d", dtype);
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
    const int bk = half_path ? HBK : BK;
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
    g.c_staged = half_path && g.out_bf16 && !g.part && !g.mask && !g.accumulate && aligned16(C) && (ldc * 2) % 16 == 0;
    dim3 grid(static_cast<unsigned>(n_wg), 1, 1);
    bool akc = !trans_a, bkc = trans_b != 0;
    if (half_path) {
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
                           const float *bias, int relu, const void *relu_mask, int64_t ldm, void *ws,
                           size_t ws_bytes, void *stream) {
    return launch_gemm(trans_a, trans_b, M, N, K, A, lda, B, ldb, C, ldc, dtype, out_f32, accumulate, bias, relu,
                       relu_mask, ldm, ws, ws_bytes, static_cast<hipStream_t>(stream));
}
