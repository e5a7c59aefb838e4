// Small VALU kernels around the layer: sigma' masking + bias gradient, softmax cross-entropy, SGD step.
#include "common.h"

#include <mutex>

#include <algorithm>

namespace capgnn {

__device__ __forceinline__ float ld_elem(const char *p, int64_t i, int bf16) {
    return bf16 ? __uint_as_float(static_cast<uint32_t>(reinterpret_cast<const uint16_t *>(p)[i]) << 16)
                : reinterpret_cast<const float *>(p)[i];
}

__device__ __forceinline__ void st_elem(char *p, int64_t i, float v, int bf16) {
    if (bf16) {
        uint32_t u = __float_as_uint(v);
        if ((u & 0x7fffffffu) > 0x7f800000u) u = (u >> 16) | 0x40u;
        else u = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
        reinterpret_cast<uint16_t *>(p)[i] = static_cast<uint16_t>(u);
    } else {
        reinterpret_cast<float *>(p)[i] = v;
    }
}

// ------------------------------------------------------------------ dZ = dH * 1[H>0], dbias partials
constexpr int RB_ROWS = 128;          // rows per chunk
constexpr int RB_MAX_BLOCKS = 1024;   // workgroups (= partial rows); each walks chunks b, b+grid, ...

// blockDim = (TX, 256/TX): threadIdx.x walks the feature columns, threadIdx.y the rows of a chunk.
// dst = src * 1[H > 0] (all of src when !relu), written in place (only the zeroed elements are stored) or,
// when dst differs from src, as a converting copy.  partial[b][f] = this workgroup's column sums of dst,
// formed from the unrounded values.
__global__ __launch_bounds__(256) void relu_mask_dbias_kernel(int64_t n, int F, const char *src, int64_t lds,
                                                              int src_bf16, char *dst, int64_t ldd, int dst_bf16,
                                                              const char *H, int64_t ldh, int h_bf16, int relu,
                                                              float *partial, const float *rscale) {
    __shared__ float red[256];
    const int tx = threadIdx.x, ty = threadIdx.y, TX = blockDim.x, TY = blockDim.y;
    const bool in_place = src == dst;
    for (int f0 = 0; f0 < F; f0 += TX) {
        const int f = f0 + tx;
        float s = 0.f;
        if (f < F) {
            for (int64_t r0 = static_cast<int64_t>(blockIdx.x) * RB_ROWS; r0 < n; r0 += static_cast<int64_t>(gridDim.x) * RB_ROWS) {
                const int64_t r1 = r0 + RB_ROWS < n ? r0 + RB_ROWS : n;
                for (int64_t r = r0 + ty; r < r1; r += TY) {
                    float g = ld_elem(src, r * lds + f, src_bf16);
                    bool zeroed = false;
                    if (relu) {
                        const float h = ld_elem(H, r * ldh + f, h_bf16);
                        if (!(h > 0.f)) { g = 0.f; zeroed = true; }
                    }
                    s += g;
                    if (rscale) g *= rscale[r];         // the stored copy carries the row's scale, the column sums do not
                    if (!in_place || zeroed || rscale) st_elem(dst, r * ldd + f, g, dst_bf16);
                }
            }
        }
        if (partial) {
            red[ty * TX + tx] = s;
            __syncthreads();
            if (ty == 0 && f < F) {
                float t = 0.f;
                for (int y = 0; y < TY; ++y) t += red[y * TX + tx];
                partial[static_cast<int64_t>(blockIdx.x) * F + f] = t;
            }
            __syncthreads();
        }
    }
}

__device__ __forceinline__ float4 ld4(const char *p, int64_t i, int bf16) {
    if (bf16) {
        const uint2 v = *reinterpret_cast<const uint2 *>(reinterpret_cast<const uint16_t *>(p) + i);
        return make_float4(__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xffff0000u), __uint_as_float(v.y << 16),
                           __uint_as_float(v.y & 0xffff0000u));
    }
    return *reinterpret_cast<const float4 *>(reinterpret_cast<const float *>(p) + i);
}

__device__ __forceinline__ uint32_t bf16_rne_bits(float v) {
    uint32_t u = __float_as_uint(v);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// The same operation with four consecutive features per thread (8- or 16-byte accesses); needs rows that start on
// 16-byte boundaries.  blockDim = (TX, 256/TX), TX = ceil(F/4) rounded up to a power of two (F <= 1024).
__global__ __launch_bounds__(256) void relu_mask_dbias_vec4_kernel(int64_t n, int F, const char *src, int64_t lds,
                                                                   int src_bf16, char *dst, int64_t ldd, int dst_bf16,
                                                                   const char *H, int64_t ldh, int h_bf16, int relu,
                                                                   float *partial, const float *rscale) {
    __shared__ float red[256][4];
    const int tx = threadIdx.x, ty = threadIdx.y, TX = blockDim.x, TY = blockDim.y;
    const bool in_place = src == dst;
    const int f = 4 * tx;
    float s[4] = {0.f, 0.f, 0.f, 0.f};
    if (f < F) {
        const int nv = F - f < 4 ? F - f : 4;    // valid features of this thread's vector (the rest is row padding)
        for (int64_t r0 = static_cast<int64_t>(blockIdx.x) * RB_ROWS; r0 < n; r0 += static_cast<int64_t>(gridDim.x) * RB_ROWS) {
            const int64_t r1 = r0 + RB_ROWS < n ? r0 + RB_ROWS : n;
            // four rows per trip: their loads are issued together, so a thread keeps eight vectors in flight
            for (int64_t rb = r0 + ty; rb < r1; rb += 4 * TY) {
                float4 gv[4], hv[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int64_t r = rb + static_cast<int64_t>(u) * TY;
                    if (r < r1) {
                        gv[u] = ld4(src, r * lds + f, src_bf16);
                        if (relu) hv[u] = ld4(H, r * ldh + f, h_bf16);
                    }
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int64_t r = rb + static_cast<int64_t>(u) * TY;
                    if (r >= r1) continue;
                    float g[4] = {gv[u].x, gv[u].y, gv[u].z, gv[u].w};
                    bool zeroed = false;
                    if (relu) {
                        const float h[4] = {hv[u].x, hv[u].y, hv[u].z, hv[u].w};
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            if (!(h[j] > 0.f) && g[j] != 0.f) { g[j] = 0.f; zeroed = true; }
                    }
#pragma unroll
                    for (int j = 0; j < 4; ++j) s[j] += g[j];
                    if (rscale) {                       // the stored copy carries the row's scale, the column sums do not
                        const float rs = rscale[r];
#pragma unroll
                        for (int j = 0; j < 4; ++j) g[j] *= rs;
                    }
                    if (!in_place || zeroed || rscale) {
                        if (nv == 4) {
                            if (dst_bf16) {
                                uint2 o;
                                o.x = bf16_rne_bits(g[0]) | (bf16_rne_bits(g[1]) << 16);
                                o.y = bf16_rne_bits(g[2]) | (bf16_rne_bits(g[3]) << 16);
                                *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(dst) + r * ldd + f) = o;
                            } else {
                                *reinterpret_cast<float4 *>(reinterpret_cast<float *>(dst) + r * ldd + f) = make_float4(g[0], g[1], g[2], g[3]);
                            }
                        } else {
                            for (int j = 0; j < nv; ++j) st_elem(dst, r * ldd + f + j, g[j], dst_bf16);
                        }
                    }
                }
            }
        }
    }
    if (!partial) return;
#pragma unroll
    for (int j = 0; j < 4; ++j) red[ty * TX + tx][j] = s[j];
    __syncthreads();
    if (ty == 0 && f < F) {
        for (int j = 0; j < 4 && f + j < F; ++j) {
            float t = 0.f;
            for (int y = 0; y < TY; ++y) t += red[y * TX + tx][j];
            partial[static_cast<int64_t>(blockIdx.x) * F + f + j] = t;
        }
    }
}

// The same for bf16 data on all three sides with eight consecutive features per thread (16-byte accesses): the wide
// bf16 layers are bound by this kernel's memory traffic, and 8-byte accesses leave half of the load path idle.
// blockDim = (TX, 256/TX), TX = ceil(F/8) rounded up to a power of two (F <= 2048); rows start on 16-byte boundaries.
__global__ __launch_bounds__(256) void relu_mask_dbias_bf16x8_kernel(int64_t n, int F, const char *src, int64_t lds, char *dst,
                                                                     int64_t ldd, const char *H, int64_t ldh, int relu,
                                                                     float *partial, const float *rscale) {
    __shared__ float red[256][8];
    const int tx = threadIdx.x, ty = threadIdx.y, TX = blockDim.x, TY = blockDim.y;
    const bool in_place = src == dst;
    const int f = 8 * tx;
    float s[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (f < F) {
        const int nv = F - f < 8 ? F - f : 8;    // valid features of this thread's vector (the rest is row padding)
        for (int64_t r0 = static_cast<int64_t>(blockIdx.x) * RB_ROWS; r0 < n; r0 += static_cast<int64_t>(gridDim.x) * RB_ROWS) {
            const int64_t r1 = r0 + RB_ROWS < n ? r0 + RB_ROWS : n;
            for (int64_t rb = r0 + ty; rb < r1; rb += 4 * TY) {
                uint4 gv[4], hv[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int64_t r = rb + static_cast<int64_t>(u) * TY;
                    if (r < r1) {
                        gv[u] = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(src) + r * lds + f);
                        if (relu) hv[u] = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(H) + r * ldh + f);
                    }
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int64_t r = rb + static_cast<int64_t>(u) * TY;
                    if (r >= r1) continue;
                    const uint32_t gw[4] = {gv[u].x, gv[u].y, gv[u].z, gv[u].w};
                    float g[8];
#pragma unroll
                    for (int d = 0; d < 4; ++d) {
                        g[2 * d] = __uint_as_float(gw[d] << 16);
                        g[2 * d + 1] = __uint_as_float(gw[d] & 0xffff0000u);
                    }
                    bool zeroed = false;
                    if (relu) {
                        const uint32_t hw[4] = {hv[u].x, hv[u].y, hv[u].z, hv[u].w};
#pragma unroll
                        for (int d = 0; d < 4; ++d) {
                            const float h0 = __uint_as_float(hw[d] << 16), h1 = __uint_as_float(hw[d] & 0xffff0000u);
                            if (!(h0 > 0.f) && g[2 * d] != 0.f) { g[2 * d] = 0.f; zeroed = true; }
                            if (!(h1 > 0.f) && g[2 * d + 1] != 0.f) { g[2 * d + 1] = 0.f; zeroed = true; }
                        }
                    }
#pragma unroll
                    for (int j = 0; j < 8; ++j) s[j] += g[j];
                    if (rscale) {                       // the stored copy carries the row's scale, the column sums do not
                        const float rs = rscale[r];
#pragma unroll
                        for (int j = 0; j < 8; ++j) g[j] *= rs;
                    }
                    if (!in_place || zeroed || rscale) {
                        if (nv == 8) {
                            uint4 o;
                            o.x = bf16_rne_bits(g[0]) | (bf16_rne_bits(g[1]) << 16);
                            o.y = bf16_rne_bits(g[2]) | (bf16_rne_bits(g[3]) << 16);
                            o.z = bf16_rne_bits(g[4]) | (bf16_rne_bits(g[5]) << 16);
                            o.w = bf16_rne_bits(g[6]) | (bf16_rne_bits(g[7]) << 16);
                            *reinterpret_cast<uint4 *>(reinterpret_cast<uint16_t *>(dst) + r * ldd + f) = o;
                        } else {
                            for (int j = 0; j < nv; ++j) st_elem(dst, r * ldd + f + j, g[j], 1);
                        }
                    }
                }
            }
        }
    }
    if (!partial) return;
#pragma unroll
    for (int j = 0; j < 8; ++j) red[ty * TX + tx][j] = s[j];
    __syncthreads();
    if (ty == 0 && f < F) {
        for (int j = 0; j < 8 && f + j < F; ++j) {
            float t = 0.f;
            for (int y = 0; y < TY; ++y) t += red[y * TX + tx][j];
            partial[static_cast<int64_t>(blockIdx.x) * F + f + j] = t;
        }
    }
}

// dbias[f] = sum_b partial[b][f]: 32 features x 32 strided groups per workgroup, doubles, fixed order
constexpr int DBF_GROUPS = 32;
__global__ __launch_bounds__(1024) void dbias_final_kernel(int64_t nblocks, int F, const float *partial, float *dbias) {
    __shared__ double red[DBF_GROUPS][32];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int f = blockIdx.x * 32 + tx;
    double s = 0.0;
    if (f < F) {
        int64_t b = ty;
        for (; b + 3 * DBF_GROUPS < nblocks; b += 4 * DBF_GROUPS) {      // four loads in flight
            const float v0 = partial[b * F + f], v1 = partial[(b + DBF_GROUPS) * F + f];
            const float v2 = partial[(b + 2 * DBF_GROUPS) * F + f], v3 = partial[(b + 3 * DBF_GROUPS) * F + f];
            s += static_cast<double>(v0); s += static_cast<double>(v1);
            s += static_cast<double>(v2); s += static_cast<double>(v3);
        }
        for (; b < nblocks; b += DBF_GROUPS) s += static_cast<double>(partial[b * F + f]);
    }
    red[ty][tx] = s;
    __syncthreads();
    if (ty == 0 && f < F) {
        double t = 0.0;
        for (int y = 0; y < DBF_GROUPS; ++y) t += red[y][tx];
        dbias[f] = static_cast<float>(t);
    }
}

static int64_t rb_blocks(int64_t n) {
    return std::max<int64_t>(1, std::min<int64_t>((n + RB_ROWS - 1) / RB_ROWS, RB_MAX_BLOCKS));
}

size_t relu_bias_ws_bytes(int64_t n, int F) {
    return align_up(static_cast<size_t>(rb_blocks(n)) * F * sizeof(float), 256);
}

int launch_relu_mask_dbias(int64_t n, int F, const void *src, int64_t lds, int src_dtype, void *dH, int64_t lddh,
                           const void *H, int64_t ldh, int dtype, int h_dtype, int relu, float *dbias, void *ws,
                           size_t ws_bytes, hipStream_t stream, const float *row_scale) {
    if (F <= 0) return CAPGNN_OK;
    if (n <= 0) {   // no rows: the bias gradient is zero (summing zero partial blocks)
        if (dbias) {
            hipLaunchKernelGGL(dbias_final_kernel, dim3((F + 31) / 32), dim3(32 * DBF_GROUPS), 0, stream, int64_t(0), F,
                               static_cast<const float *>(nullptr), dbias);
            CG_HIP(hipGetLastError());
        }
        return CAPGNN_OK;
    }
    if (!src) { src = dH; lds = lddh; src_dtype = dtype; }
    const bool converting = src != dH;
    if (!relu && !dbias && !converting && !row_scale) return CAPGNN_OK;
    if (!dH || (relu && !H)) CG_FAIL(CAPGNN_EINVAL, "relu_mask_dbias: NULL operand");
    if (lddh < F || lds < F || (relu && ldh < F)) CG_FAIL(CAPGNN_EINVAL, "relu_mask_dbias: leading dimension smaller than F");
    const int64_t nb = rb_blocks(n);
    if (dbias && (!ws || ws_bytes < static_cast<size_t>(nb) * F * sizeof(float)))
        CG_FAIL(CAPGNN_ENOMEM, "relu_mask_dbias: workspace too small");
    const int ses = elem_bytes(src_dtype), des = elem_bytes(dtype), hes = elem_bytes(h_dtype);
    const bool vec = F <= 1024 && aligned16(src) && aligned16(dH) && (lds * ses) % 16 == 0 && (lddh * des) % 16 == 0 &&
                     (!relu || (aligned16(H) && (ldh * hes) % 16 == 0));
    const bool all_bf16 = src_dtype == CAPGNN_BF16 && dtype == CAPGNN_BF16 && (!relu || h_dtype == CAPGNN_BF16);
    if (vec && all_bf16 && F >= 64 && F <= 2048) {
        int TX = 1;
        while (TX < (F + 7) / 8) TX <<= 1;
        dim3 block(TX, 256 / TX);
        hipLaunchKernelGGL(relu_mask_dbias_bf16x8_kernel, dim3(static_cast<unsigned>(nb)), block, 0, stream, n, F,
                           static_cast<const char *>(src), lds, static_cast<char *>(dH), lddh, static_cast<const char *>(H), ldh,
                           relu, dbias ? static_cast<float *>(ws) : nullptr, row_scale);
        CG_HIP(hipGetLastError());
        if (dbias) {
            hipLaunchKernelGGL(dbias_final_kernel, dim3((F + 31) / 32), dim3(32 * DBF_GROUPS), 0, stream, nb, F,
                               static_cast<const float *>(ws), dbias);
            CG_HIP(hipGetLastError());
        }
        return CAPGNN_OK;
    }
    if (vec) {
        int TX = 1;
        while (TX < (F + 3) / 4) TX <<= 1;
        dim3 block(TX, 256 / TX);
        hipLaunchKernelGGL(relu_mask_dbias_vec4_kernel, dim3(static_cast<unsigned>(nb)), block, 0, stream, n, F,
                           static_cast<const char *>(src), lds, src_dtype == CAPGNN_BF16 ? 1 : 0, static_cast<char *>(dH), lddh,
                           dtype == CAPGNN_BF16 ? 1 : 0, static_cast<const char *>(H), ldh, h_dtype == CAPGNN_BF16 ? 1 : 0,
                           relu, dbias ? static_cast<float *>(ws) : nullptr, row_scale);
        CG_HIP(hipGetLastError());
        if (dbias) {
            hipLaunchKernelGGL(dbias_final_kernel, dim3((F + 31) / 32), dim3(32 * DBF_GROUPS), 0, stream, nb, F,
                               static_cast<const float *>(ws), dbias);
            CG_HIP(hipGetLastError());
        }
        return CAPGNN_OK;
    }
    int TX = 1;
    while (TX < F && TX < 256) TX <<= 1;
    dim3 block(TX, 256 / TX);
    hipLaunchKernelGGL(relu_mask_dbias_kernel, dim3(static_cast<unsigned>(nb)), block, 0, stream, n, F,
                       static_cast<const char *>(src), lds, src_dtype == CAPGNN_BF16 ? 1 : 0, static_cast<char *>(dH), lddh,
                       dtype == CAPGNN_BF16 ? 1 : 0, static_cast<const char *>(H), ldh, h_dtype == CAPGNN_BF16 ? 1 : 0,
                       relu, dbias ? static_cast<float *>(ws) : nullptr, row_scale);
    CG_HIP(hipGetLastError());
    if (dbias) {
        hipLaunchKernelGGL(dbias_final_kernel, dim3((F + 31) / 32), dim3(32 * DBF_GROUPS), 0, stream, nb, F,
                           static_cast<const float *>(ws), dbias);
        CG_HIP(hipGetLastError());
    }
    return CAPGNN_OK;
}

// ------------------------------------------------------------------ SGD
__global__ __launch_bounds__(256) void sgd_kernel(float *W, const float *dW, int64_t n, float lr) {
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; i < n;
         i += static_cast<int64_t>(gridDim.x) * 256)
        W[i] = W[i] - lr * dW[i];
}

int launch_sgd(float *W, const float *dW, int64_t n, float lr, hipStream_t stream) {
    if (n <= 0) return CAPGNN_OK;
    if (!W || !dW) CG_FAIL(CAPGNN_EINVAL, "sgd: NULL operand");
    const unsigned blocks = static_cast<unsigned>(std::min<int64_t>((n + 255) / 256, 2048));
    hipLaunchKernelGGL(sgd_kernel, dim3(blocks), dim3(256), 0, stream, W, dW, n, lr);
    CG_HIP(hipGetLastError());
    return CAPGNN_OK;
}

// ------------------------------------------------------------------ masked softmax cross-entropy
// scratch layout (bytes): [0] normaliser (float); [256, 256 + 8*LOSS_PARTS) per-workgroup partial sums (double);
// [LOSS_HEADER ..] per-row loss terms (float).  Both reductions are two-level with fixed summation orders.
constexpr int LOSS_PARTS = 512;
constexpr size_t LOSS_HEADER = 8192;

__device__ __forceinline__ double block_sum_1024(double c, double *red) {
    red[threadIdx.x] = c;
    __syncthreads();
    for (int s = 512; s > 0; s >>= 1) {
        if (threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
        __syncthreads();
    }
    return red[0];
}

// part[b] = number of masked rows in workgroup b's contiguous slice
__global__ __launch_bounds__(1024) void count_mask_kernel(int64_t n, const uint8_t *mask, double *part) {
    __shared__ double red[1024];
    const int64_t per = (n + gridDim.x - 1) / gridDim.x;
    const int64_t lo = blockIdx.x * per, hi = lo + per < n ? lo + per : n;
    double c = 0.0;
    for (int64_t i = lo + threadIdx.x; i < hi; i += 1024) c += mask[i] ? 1.0 : 0.0;
    c = block_sum_1024(c, red);
    if (threadIdx.x == 0) part[blockIdx.x] = c;
}

__global__ __launch_bounds__(64) void count_final_kernel(int parts, const double *part, float times, float *norm_out) {
    if (threadIdx.x != 0) return;
    double c = 0.0;
    for (int b = 0; b < parts; ++b) c += part[b];
    norm_out[0] = (c > 0.0 ? static_cast<float>(c) : 1.f) * times;
}

// A group of lpr lanes (a power of two, 4..64, about a quarter of the classes) per row, so that narrow class counts
// still keep 64/lpr rows in flight per wave; the lanes of a group stride over the classes.
static int loss_lanes_per_row_host(int C) {
    int lpr = 4;
    while (lpr < 64 && lpr * 4 < C) lpr *= 2;
    return lpr;
}

// One lane group (lpr lanes) per row.  A lane's logits (classes l, l + lpr, ...) are read once and kept: up to four per
// lane in registers, which covers every C <= 4 * lpr (all C <= 256); beyond that the row is read again from the L1.
// One exponential per class: the terms of the sum are reused for the gradient, p_k = e_k / s.  copy: when not null, the
// logits are also written there as a dense [n x C] matrix (what the caller of an epoch asked for as `logits`).
__global__ __launch_bounds__(256) void softmax_ce_kernel(int64_t n, int C, int lpr, const float *Z, int64_t ldz,
                                                         const int32_t *labels, const uint8_t *mask, float norm_val,
                                                         const float *norm_dev, float *row_loss, char *dZ,
                                                         int64_t lddz, int dz_bf16, float *copy) {
    const int lane = threadIdx.x & 63;
    const int l = lane % lpr;
    const int64_t row = (static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6)) * (64 / lpr) + lane / lpr;
    if (row >= n) return;          // whole lane groups leave; the shuffles below stay inside a group
    const float norm = norm_dev ? norm_dev[0] : norm_val;
    const bool on = !mask || mask[row];
    const float *z = Z + row * ldz;
    constexpr int KEEP = 4;
    float zr[KEEP];
#pragma unroll
    for (int j = 0; j < KEEP; ++j) {
        const int k = l + j * lpr;
        zr[j] = k < C ? z[k] : -INFINITY;
        if (copy && k < C) copy[row * C + k] = zr[j];
    }
    const bool kept = C <= KEEP * lpr;
    if (copy && !kept) for (int k = l + KEEP * lpr; k < C; k += lpr) copy[row * C + k] = z[k];
    if (!on) {
        if (l == 0) row_loss[row] = 0.f;
        if (dZ) for (int k = l; k < C; k += lpr) st_elem(dZ, row * lddz + k, 0.f, dz_bf16);
        return;
    }
    float m = fmaxf(fmaxf(zr[0], zr[1]), fmaxf(zr[2], zr[3]));
    if (!kept) for (int k = l + KEEP * lpr; k < C; k += lpr) m = fmaxf(m, z[k]);
    for (int off = lpr >> 1; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    float er[KEEP];
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < KEEP; ++j) {
        er[j] = (l + j * lpr < C) ? expf(zr[j] - m) : 0.f;
        s += er[j];
    }
    if (!kept) for (int k = l + KEEP * lpr; k < C; k += lpr) s += expf(z[k] - m);
    for (int off = lpr >> 1; off > 0; off >>= 1) s += __shfl_xor(s, off);
    const float lse = m + logf(s);
    int y = labels[row];
    y = y < 0 ? 0 : (y >= C ? C - 1 : y);
    if (l == 0) row_loss[row] = lse - z[y];
    if (dZ) {
        const float inv = 1.f / norm, inv_s = 1.f / s;
#pragma unroll
        for (int j = 0; j < KEEP; ++j) {
            const int k = l + j * lpr;
            if (k < C) st_elem(dZ, row * lddz + k, (er[j] * inv_s - (k == y ? 1.f : 0.f)) * inv, dz_bf16);
        }
        if (!kept)
            for (int k = l + KEEP * lpr; k < C; k += lpr)
                st_elem(dZ, row * lddz + k, (expf(z[k] - m) * inv_s - (k == y ? 1.f : 0.f)) * inv, dz_bf16);
    }
}

// Binary cross-entropy on logits, one lane group per row like the softmax kernel: the element's loss in the form
// max(z,0) - z*y + log(1 + exp(-|z|)), which neither overflows nor cancels, and its derivative s(z) - y.
__global__ __launch_bounds__(256) void sigmoid_bce_kernel(int64_t n, int C, int lpr, const float *Z, int64_t ldz,
                                                          const uint8_t *targets, int64_t ldt, const uint8_t *mask,
                                                          float norm_val, const float *norm_dev, float *row_loss, char *dZ,
                                                          int64_t lddz, int dz_bf16) {
    const int lane = threadIdx.x & 63;
    const int l = lane % lpr;
    const int64_t row = (static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6)) * (64 / lpr) + lane / lpr;
    if (row >= n) return;
    const bool on = !mask || mask[row];
    if (!on) {
        if (l == 0) row_loss[row] = 0.f;
        if (dZ) for (int k = l; k < C; k += lpr) st_elem(dZ, row * lddz + k, 0.f, dz_bf16);
        return;
    }
    const float inv = 1.f / (norm_dev ? norm_dev[0] : norm_val);
    const float *z = Z + row * ldz;
    const uint8_t *t = targets + row * ldt;
    float s = 0.f;
    for (int k = l; k < C; k += lpr) {
        const float zk = z[k], y = t[k] ? 1.f : 0.f;
        const float e = expf(-fabsf(zk));
        s += fmaxf(zk, 0.f) - zk * y + log1pf(e);
        if (dZ) {
            const float sig = zk >= 0.f ? 1.f / (1.f + e) : e / (1.f + e);
            st_elem(dZ, row * lddz + k, (sig - y) * inv, dz_bf16);
        }
    }
    for (int off = lpr >> 1; off > 0; off >>= 1) s += __shfl_xor(s, off);
    if (l == 0) row_loss[row] = s;
}

__global__ __launch_bounds__(1024) void loss_partial_kernel(int64_t n, const float *row_loss, double *part) {
    __shared__ double red[1024];
    const int64_t per = (n + gridDim.x - 1) / gridDim.x;
    const int64_t lo = blockIdx.x * per, hi = lo + per < n ? lo + per : n;
    double c = 0.0;
    for (int64_t i = lo + threadIdx.x; i < hi; i += 1024) c += static_cast<double>(row_loss[i]);
    c = block_sum_1024(c, red);
    if (threadIdx.x == 0) part[blockIdx.x] = c;
}

__global__ __launch_bounds__(64) void loss_final_kernel(int parts, const double *part, float norm_val, const float *norm_dev,
                                                        float *loss_out) {
    if (threadIdx.x != 0) return;
    double c = 0.0;
    for (int b = 0; b < parts; ++b) c += part[b];
    const double norm = norm_dev ? static_cast<double>(norm_dev[0]) : static_cast<double>(norm_val);
    loss_out[0] = static_cast<float>(c / norm);
}

// Up to LOSS_SMALL_N rows: one workgroup does a whole reduction (16-byte loads, fixed order), which saves the second
// launch of the two-level form; these kernels run for a few microseconds either way.
constexpr int64_t LOSS_SMALL_N = int64_t(1) << 18;

__device__ __forceinline__ int nonzero_bytes(uint32_t w) {
    return ((w & 0xffu) != 0) + ((w & 0xff00u) != 0) + ((w & 0xff0000u) != 0) + ((w & 0xff000000u) != 0);
}

// norm_out[0] = max(number of masked rows, 1) * times; mask must start on a 16-byte boundary
__global__ __launch_bounds__(1024) void count_small_kernel(int64_t n, const uint8_t *mask, float times, float *norm_out) {
    __shared__ double red[1024];
    const int64_t n16 = n / 16;
    const uint4 *m4 = reinterpret_cast<const uint4 *>(mask);
    int cnt = 0;
    for (int64_t i = threadIdx.x; i < n16; i += 1024) {
        const uint4 v = m4[i];
        cnt += nonzero_bytes(v.x) + nonzero_bytes(v.y) + nonzero_bytes(v.z) + nonzero_bytes(v.w);
    }
    for (int64_t i = n16 * 16 + threadIdx.x; i < n; i += 1024) cnt += mask[i] ? 1 : 0;
    const double c = block_sum_1024(static_cast<double>(cnt), red);
    if (threadIdx.x == 0) norm_out[0] = (c > 0.0 ? static_cast<float>(c) : 1.f) * times;
}

// loss_out[0] = sum(row_loss) / norm; row_loss must start on a 16-byte boundary
__global__ __launch_bounds__(1024) void loss_small_kernel(int64_t n, const float *row_loss, float norm_val, const float *norm_dev,
                                                          float *loss_out) {
    __shared__ double red[1024];
    const int64_t n4 = n / 4;
    const float4 *r4 = reinterpret_cast<const float4 *>(row_loss);
    double c = 0.0;
    for (int64_t i = threadIdx.x; i < n4; i += 1024) {
        const float4 v = r4[i];
        c += static_cast<double>(v.x); c += static_cast<double>(v.y); c += static_cast<double>(v.z); c += static_cast<double>(v.w);
    }
    for (int64_t i = n4 * 4 + threadIdx.x; i < n; i += 1024) c += static_cast<double>(row_loss[i]);
    c = block_sum_1024(c, red);
    if (threadIdx.x == 0) {
        const double norm = norm_dev ? static_cast<double>(norm_dev[0]) : static_cast<double>(norm_val);
        loss_out[0] = static_cast<float>(c / norm);
    }
}

// the two reductions around a loss kernel: the normaliser from the mask, and the loss from the per-row terms
static void launch_mask_count(int64_t n, const uint8_t *mask, float times, double *part, int parts, float *norm_dev,
                              hipStream_t st) {
    if (n <= LOSS_SMALL_N && reinterpret_cast<uintptr_t>(mask) % 16 == 0) {
        hipLaunchKernelGGL(count_small_kernel, dim3(1), dim3(1024), 0, st, n, mask, times, norm_dev);
        return;
    }
    hipLaunchKernelGGL(count_mask_kernel, dim3(parts), dim3(1024), 0, st, n, mask, part);
    hipLaunchKernelGGL(count_final_kernel, dim3(1), dim3(64), 0, st, parts, part, times, norm_dev);
}

static void launch_loss_sum(int64_t n, const float *row_loss, double *part, int parts, float norm_val, const float *norm_dev,
                            float *loss_dev, hipStream_t st) {
    if (n <= LOSS_SMALL_N && reinterpret_cast<uintptr_t>(row_loss) % 16 == 0) {
        hipLaunchKernelGGL(loss_small_kernel, dim3(1), dim3(1024), 0, st, n, row_loss, norm_val, norm_dev, loss_dev);
        return;
    }
    hipLaunchKernelGGL(loss_partial_kernel, dim3(parts), dim3(1024), 0, st, n, row_loss, part);
    hipLaunchKernelGGL(loss_final_kernel, dim3(1), dim3(64), 0, st, parts, part, norm_val, norm_dev, loss_dev);
}

}  // namespace capgnn

using namespace capgnn;

extern "C" size_t capgnn_loss_workspace_bytes(int64_t n) {
    return align_up(LOSS_HEADER + static_cast<size_t>(n > 0 ? n : 1) * sizeof(float), 256);
}

extern "C" int capgnn_sigmoid_bce(int64_t n, int C, const float *Z, int64_t ldz, const uint8_t *targets, int64_t ldt,
                                  const uint8_t *mask, double loss_norm, float *loss_dev, void *dZ, int64_t lddz,
                                  int dz_dtype, void *ws, size_t ws_bytes, void *stream) {
    if (dz_dtype != CAPGNN_F32 && dz_dtype != CAPGNN_BF16) CG_FAIL(CAPGNN_EINVAL, "sigmoid_bce: unknown dz_dtype");
    if (n < 0 || C <= 0) CG_FAIL(CAPGNN_EINVAL, "sigmoid_bce: bad sizes");
    if (n == 0) return CAPGNN_OK;
    if (!Z || !targets || !loss_dev) CG_FAIL(CAPGNN_EINVAL, "sigmoid_bce: NULL operand");
    if (ldz < C || ldt < C || (dZ && lddz < C)) CG_FAIL(CAPGNN_EINVAL, "sigmoid_bce: leading dimension smaller than C");
    if (!ws || ws_bytes < capgnn_loss_workspace_bytes(n)) CG_FAIL(CAPGNN_ENOMEM, "sigmoid_bce: workspace too small");
    hipStream_t st = static_cast<hipStream_t>(stream);
    float *norm_dev = nullptr;
    float norm_val = 1.f;
    double *part = reinterpret_cast<double *>(static_cast<char *>(ws) + 256);
    const int parts = static_cast<int>(std::max<int64_t>(1, std::min<int64_t>((n + 4095) / 4096, LOSS_PARTS)));
    if (loss_norm > 0.0) norm_val = static_cast<float>(loss_norm);
    else if (!mask) norm_val = static_cast<float>(n) * static_cast<float>(C);
    else {   // masked rows x classes
        norm_dev = static_cast<float *>(ws);
        launch_mask_count(n, mask, static_cast<float>(C), part, parts, norm_dev, st);
    }
    float *row_loss = reinterpret_cast<float *>(static_cast<char *>(ws) + LOSS_HEADER);
    const int lpr = loss_lanes_per_row_host(C);
    const int64_t rows_per_block = 4 * (64 / lpr);
    hipLaunchKernelGGL(sigmoid_bce_kernel, dim3(static_cast<unsigned>((n + rows_per_block - 1) / rows_per_block)), dim3(256), 0, st, n, C, lpr, Z, ldz, targets,
                       ldt, mask, norm_val, norm_dev, row_loss, static_cast<char *>(dZ), lddz, dz_dtype == CAPGNN_BF16 ? 1 : 0);
    launch_loss_sum(n, row_loss, part, parts, norm_val, norm_dev, loss_dev, st);
    CG_HIP(hipGetLastError());
    return CAPGNN_OK;
}

// everything capgnn_softmax_ce does after its argument checks; `ws` holds capgnn_loss_workspace_bytes(n) bytes
static int softmax_ce_launch(int64_t n, int C, const float *Z, int64_t ldz, const int32_t *labels, const uint8_t *mask,
                             double loss_norm, float *loss_dev, void *dZ, int64_t lddz, int dz_dtype, void *ws,
                             hipStream_t st, float *copy = nullptr) {
    float *norm_dev = nullptr;
    float norm_val = 1.f;
    float *scratch = static_cast<float *>(ws);
    double *part = reinterpret_cast<double *>(static_cast<char *>(ws) + 256);
    const int parts = static_cast<int>(std::max<int64_t>(1, std::min<int64_t>((n + 4095) / 4096, LOSS_PARTS)));
    if (loss_norm > 0.0) norm_val = static_cast<float>(loss_norm);
    else if (!mask) norm_val = static_cast<float>(n);
    else {
        norm_dev = scratch;
        launch_mask_count(n, mask, 1.f, part, parts, norm_dev, st);
    }
    float *row_loss = reinterpret_cast<float *>(static_cast<char *>(ws) + LOSS_HEADER);
    const int lpr = loss_lanes_per_row_host(C);
    const int64_t rows_per_block = 4 * (64 / lpr);
    hipLaunchKernelGGL(softmax_ce_kernel, dim3(static_cast<unsigned>((n + rows_per_block - 1) / rows_per_block)), dim3(256), 0, st, n, C, lpr, Z, ldz,
                       labels, mask, norm_val, norm_dev, row_loss, static_cast<char *>(dZ), lddz, dz_dtype == CAPGNN_BF16 ? 1 : 0, copy);
    launch_loss_sum(n, row_loss, part, parts, norm_val, norm_dev, loss_dev, st);
    CG_HIP(hipGetLastError());
    return CAPGNN_OK;
}

static int softmax_ce_check(int64_t n, int C, const float *Z, int64_t ldz, const int32_t *labels, float *loss_dev,
                            const void *dZ, int64_t lddz, int dz_dtype) {
    if (dz_dtype != CAPGNN_F32 && dz_dtype != CAPGNN_BF16) CG_FAIL(CAPGNN_EINVAL, "softmax_ce: unknown dz_dtype");
    if (n < 0 || C <= 0) CG_FAIL(CAPGNN_EINVAL, "softmax_ce: bad sizes");
    if (n == 0) return CAPGNN_OK;
    if (!Z || !labels || !loss_dev) CG_FAIL(CAPGNN_EINVAL, "softmax_ce: NULL operand");
    if (ldz < C || (dZ && lddz < C)) CG_FAIL(CAPGNN_EINVAL, "softmax_ce: leading dimension smaller than C");
    return CAPGNN_OK;
}

extern "C" int capgnn_softmax_ce(int64_t n, int C, const float *Z, int64_t ldz, const int32_t *labels,
                                 const uint8_t *mask, double loss_norm, float *loss_dev, void *dZ, int64_t lddz,
                                 int dz_dtype, void *ws, size_t ws_bytes, void *stream) {
    CG_TRY(softmax_ce_check(n, C, Z, ldz, labels, loss_dev, dZ, lddz, dz_dtype));
    if (n == 0) return CAPGNN_OK;
    if (!ws || ws_bytes < capgnn_loss_workspace_bytes(n)) CG_FAIL(CAPGNN_ENOMEM, "softmax_ce: workspace too small");
    return softmax_ce_launch(n, C, Z, ldz, labels, mask, loss_norm, loss_dev, dZ, lddz, dz_dtype, ws,
                             static_cast<hipStream_t>(stream));
}

// capgnn_softmax_ce for the epoch, which also wants the logits as a dense [n x C] copy (or not: copy may be NULL)
int capgnn::softmax_ce_with_copy(int64_t n, int C, const float *Z, int64_t ldz, const int32_t *labels, const uint8_t *mask,
                         double loss_norm, float *loss_dev, void *dZ, int64_t lddz, int dz_dtype, void *ws, size_t ws_bytes,
                         hipStream_t st, float *copy) {
    CG_TRY(softmax_ce_check(n, C, Z, ldz, labels, loss_dev, dZ, lddz, dz_dtype));
    if (n == 0) return CAPGNN_OK;
    if (!ws || ws_bytes < capgnn_loss_workspace_bytes(n)) CG_FAIL(CAPGNN_ENOMEM, "softmax_ce: workspace too small");
    return softmax_ce_launch(n, C, Z, ldz, labels, mask, loss_norm, loss_dev, dZ, lddz, dz_dtype, ws, st, copy);
}

// ------------------------------------------------------------------ the same loss without any allocation by anyone
// The scratch of capgnn_softmax_ce (normaliser, per-workgroup partial sums, per-row loss terms) for up to
// CAPGNN_LOSS_STATIC_MAX_ROWS rows, as a device array that is part of the library image: every GPU the library
// runs on holds its own copy until the process ends.  Host code never uses the array's name as an address: the
// address on the current device is asked for once per device and kept.
static __device__ __align__(256) unsigned char scratch[LOSS_HEADER + static_cast<size_t>(CAPGNN_LOSS_STATIC_MAX_ROWS) * sizeof(float)];

constexpr int MAX_DEVICES = 64;
static void *g_scratch_ptr[MAX_DEVICES];
static std::mutex g_scratch_mutex;

// device address of `scratch` on the current device (looked up on the first call on that device)
static int static_scratch(void **out) {
    int dev = -1;
    CG_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) CG_FAIL(CAPGNN_EUNSUPPORTED, "softmax_ce_static: device ordinal %d out of range", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        CG_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) CG_FAIL(CAPGNN_EHIP, "softmax_ce_static: the scratch array has no address on device %d", dev);
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return CAPGNN_OK;
}

extern "C" int capgnn_softmax_ce_static(int64_t n, int C, const float *Z, int64_t ldz, const int32_t *labels,
                                        const uint8_t *mask, double loss_norm, float *loss_dev, void *dZ, int64_t lddz,
                                        int dz_dtype, void *stream) {
    CG_TRY(softmax_ce_check(n, C, Z, ldz, labels, loss_dev, dZ, lddz, dz_dtype));
    if (n > CAPGNN_LOSS_STATIC_MAX_ROWS)
        CG_FAIL(CAPGNN_ENOMEM, "softmax_ce_static: %lld rows, the built-in scratch holds %d; use capgnn_softmax_ce with a workspace",
                static_cast<long long>(n), CAPGNN_LOSS_STATIC_MAX_ROWS);
    if (n == 0) return CAPGNN_OK;
    void *ws = nullptr;
    CG_TRY(static_scratch(&ws));
    // nothing in the scratch has to start at zero: the normaliser, parts[0..parts) and row terms [0, n) are all written
    // before they are read, so what an earlier (larger) call left behind is never seen
    return softmax_ce_launch(n, C, Z, ldz, labels, mask, loss_norm, loss_dev, dZ, lddz, dz_dtype, ws,
                             static_cast<hipStream_t>(stream));
}
