// Two-tier halo cache: placement, id -> (tier, slot) maps, lookup and the row gather.
//
// GPU tier = rows in device memory, host tier = rows in pinned host memory.  Placement ranks the
// halo vertices by (priority descending, global id ascending).  Within a tier, slots are numbered
// in ascending halo-local order so that the full-batch gather walks both the table and the
// destination buffer monotonically.  The gather itself is a plain row copy: 16-byte lanes, several
// rows per wave when rows are short, no arithmetic on the data (results are bit copies).
#include "common.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <numeric>

namespace capgnn {

__host__ __device__ inline uint64_t mix64(uint64_t x) {
    x += 0x9e3779b97f4a7c15ull;
    x = (x ^ (x >> 30)) * 0xbf58476d1ce4e5b9ull;
    x = (x ^ (x >> 27)) * 0x94d049bb133111ebull;
    return x ^ (x >> 31);
}

uint64_t hash_gid(uint64_t x) { return mix64(x); }

struct MapView {
    int64_t n_halo;
    const int32_t *slot;      // [n_halo]
    const int64_t *hkeys;     // hash keys or null
    const int32_t *hvals;
    uint64_t hmask;
};

// halo-local index of a request id, or -1
__host__ __device__ inline int64_t resolve(const MapView &m, int64_t id, int by_gid) {
    if (!by_gid) return (id >= 0 && id < m.n_halo) ? id : -1;
    if (!m.hkeys) return -1;
    uint64_t p = mix64(static_cast<uint64_t>(id)) & m.hmask;
    for (uint64_t probes = 0; probes <= m.hmask; ++probes) {
        const int32_t v = m.hvals[p];
        if (v < 0) return -1;
        if (m.hkeys[p] == id) return v;
        p = (p + 1) & m.hmask;
    }
    return -1;
}

__global__ __launch_bounds__(256) void lookup_kernel(MapView m, const int64_t *ids, int64_t n, int by_gid,
                                                     int8_t *tier, int64_t *slot) {
    const int64_t k = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (k >= n) return;
    const int64_t h = resolve(m, ids[k], by_gid);
    if (h < 0) {
        tier[k] = -1;
        slot[k] = -1;
    } else {
        const int32_t s = m.slot[h];
        tier[k] = s >= 0 ? 0 : 1;
        slot[k] = s >= 0 ? s : -1 - static_cast<int64_t>(s);
    }
}

// copies row_bytes bytes from s to d with the lanes l, l+lpr, ... of one lane group
__device__ __forceinline__ void copy_row(const char *s, char *d, int row_bytes, int l, int lpr, int vec16, int es) {
    int done = 0;
    if (vec16) {
        const int nfull = row_bytes >> 4;
        const uint4 *sv = reinterpret_cast<const uint4 *>(s);
        uint4 *dv = reinterpret_cast<uint4 *>(d);
        int c = l;
        for (; c + 3 * lpr < nfull; c += 4 * lpr) {
            const uint4 a0 = sv[c], a1 = sv[c + lpr], a2 = sv[c + 2 * lpr], a3 = sv[c + 3 * lpr];
            dv[c] = a0; dv[c + lpr] = a1; dv[c + 2 * lpr] = a2; dv[c + 3 * lpr] = a3;
        }
        for (; c < nfull; c += lpr) dv[c] = sv[c];
        done = nfull << 4;
    }
    if (es == 4) {
        for (int b = done + l * 4; b < row_bytes; b += lpr * 4)
            *reinterpret_cast<uint32_t *>(d + b) = *reinterpret_cast<const uint32_t *>(s + b);
    } else {
        for (int b = done + l * 2; b < row_bytes; b += lpr * 2)
            *reinterpret_cast<uint16_t *>(d + b) = *reinterpret_cast<const uint16_t *>(s + b);
    }
}

__device__ __forceinline__ void zero_row(char *d, int row_bytes, int l, int lpr, int es) {
    if (es == 4) for (int b = l * 4; b < row_bytes; b += lpr * 4) *reinterpret_cast<uint32_t *>(d + b) = 0u;
    else for (int b = l * 2; b < row_bytes; b += lpr * 2) *reinterpret_cast<uint16_t *>(d + b) = 0;
}

// out[dst_list[k]] = table[k]  (full-batch gather of one tier; dst_list = halo-local index of slot k).
// A lane group moves SCATTER_ROWS rows at a time: their destination indices are fetched together, then one 16-byte
// load per row is issued before the first store, so that a wave keeps several kilobytes in flight even when a row
// is a single load wide (the copy is latency-bound otherwise: index, row, store are three dependent round trips).
constexpr int SCATTER_ROWS = 4;

// One tier's rows and where they go; `blocks` workgroups of the launch work on it.
struct TierRows {
    const char *table;
    const int32_t *dst_list;
    int64_t n;
    unsigned blocks;
};

// One launch serves up to two tiers of the same layer (same pitch and row geometry): workgroups [0, a.blocks) take
// tier a, the rest tier b.
__global__ __launch_bounds__(256) void scatter_tier_kernel(TierRows a, TierRows b, int64_t pitch, char *out,
                                                           int64_t out_pitch, int row_bytes, int lpr, int vec16, int es) {
    const bool second = blockIdx.x >= a.blocks;            // uniform over the workgroup
    const char *table = second ? b.table : a.table;
    const int32_t *dst_list = second ? b.dst_list : a.dst_list;
    const int64_t n = second ? b.n : a.n;
    const unsigned blocks = second ? b.blocks : a.blocks;
    const unsigned bx = second ? blockIdx.x - a.blocks : blockIdx.x;
    const int lane = threadIdx.x & 63;
    const int l = lane % lpr;
    const int rows_per_wave = 64 / lpr;
    const int64_t wave = static_cast<int64_t>(bx) * 4 + (threadIdx.x >> 6);
    const int64_t per_wave = static_cast<int64_t>(rows_per_wave) * SCATTER_ROWS;
    const int64_t stride = static_cast<int64_t>(blocks) * 4 * per_wave;   // a capped grid walks the list in strides
    for (int64_t base = wave * per_wave; base < n; base += stride) {
        const int64_t k0 = base + lane / lpr;
        const char *src[SCATTER_ROWS];
        char *dst[SCATTER_ROWS];
        int32_t di[SCATTER_ROWS];
#pragma unroll
        for (int u = 0; u < SCATTER_ROWS; ++u) {
            const int64_t k = k0 + static_cast<int64_t>(u) * rows_per_wave;
            di[u] = k < n ? dst_list[k] : -1;
        }
#pragma unroll
        for (int u = 0; u < SCATTER_ROWS; ++u) {
            const int64_t k = k0 + static_cast<int64_t>(u) * rows_per_wave;
            src[u] = table + k * pitch;
            dst[u] = out + static_cast<int64_t>(di[u]) * out_pitch;
        }
        int done = 0;
        if (vec16) {
            const int nfull = row_bytes >> 4;
            for (int c = l; c < nfull; c += lpr) {
                uint4 a[SCATTER_ROWS];
#pragma unroll
                for (int u = 0; u < SCATTER_ROWS; ++u)
                    if (di[u] >= 0) a[u] = reinterpret_cast<const uint4 *>(src[u])[c];
#pragma unroll
                for (int u = 0; u < SCATTER_ROWS; ++u)
                    if (di[u] >= 0) reinterpret_cast<uint4 *>(dst[u])[c] = a[u];
            }
            done = nfull << 4;
        }
        if (done < row_bytes) {   // the last few elements of a row, or rows that are not 16-byte aligned
#pragma unroll
            for (int u = 0; u < SCATTER_ROWS; ++u) {
                if (di[u] < 0) continue;
                if (es == 4) {
                    for (int b = done + l * 4; b < row_bytes; b += lpr * 4)
                        *reinterpret_cast<uint32_t *>(dst[u] + b) = *reinterpret_cast<const uint32_t *>(src[u] + b);
                } else {
                    for (int b = done + l * 2; b < row_bytes; b += lpr * 2)
                        *reinterpret_cast<uint16_t *>(dst[u] + b) = *reinterpret_cast<const uint16_t *>(src[u] + b);
                }
            }
        }
    }
}

// request-list gather with lookup; which: bit0 = serve GPU-tier rows (and absent ids), bit1 = serve host-tier rows
__global__ __launch_bounds__(256) void gather_ids_kernel(MapView m, const int64_t *ids, int64_t n, int by_gid,
                                                         const char *gpu_table, const char *host_table, int64_t pitch,
                                                         int which, char *out, int64_t out_pitch, int row_bytes,
                                                         int lpr, int vec16, int es, unsigned long long *counters) {
    const int lane = threadIdx.x & 63;
    const int64_t wave = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    const int64_t k = wave * (64 / lpr) + lane / lpr;
    if (k >= n) return;
    const int l = lane % lpr;
    const int64_t h = resolve(m, ids[k], by_gid);
    char *d = out + k * out_pitch;
    if (h < 0) {
        if (which & 1) {
            zero_row(d, row_bytes, l, lpr, es);
            if (counters && l == 0) atomicAdd(&counters[2], 1ull);
        }
        return;
    }
    const int32_t s = m.slot[h];
    if (s >= 0) {
        if (which & 1) {
            copy_row(gpu_table + static_cast<int64_t>(s) * pitch, d, row_bytes, l, lpr, vec16, es);
            if (counters && l == 0) atomicAdd(&counters[0], 1ull);
        }
    } else if (which & 2) {
        copy_row(host_table + (-1 - static_cast<int64_t>(s)) * pitch, d, row_bytes, l, lpr, vec16, es);
        if (counters && l == 0) atomicAdd(&counters[1], 1ull);
    }
}

// ---- vertex update.  Pass 1 finds, for every vertex named in the call, the position of its last update;
// pass 2 lets exactly that position write the row, then the stamp, and clears the scratch again.
__global__ __launch_bounds__(256) void update_owner_kernel(MapView m, const int64_t *ids, int64_t n, int by_gid,
                                                           long long *owner) {
    const int64_t k = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (k >= n) return;
    const int64_t h = resolve(m, ids[k], by_gid);
    if (h >= 0) atomicMax(&owner[h], static_cast<long long>(k));
}

__global__ __launch_bounds__(256) void update_rows_kernel(MapView m, const int64_t *ids, int64_t n, int by_gid,
                                                          const char *rows, int64_t rows_pitch, char *gpu_table,
                                                          char *host_table, char *staged_table, int64_t pitch,
                                                          int row_bytes, int lpr, int vec16, int es, const long long *owner,
                                                          int64_t *stamp, int64_t epoch, unsigned long long *counters) {
    const int lane = threadIdx.x & 63;
    const int64_t wave = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    const int64_t k = wave * (64 / lpr) + lane / lpr;
    if (k >= n) return;
    const int l = lane % lpr;
    const int64_t h = resolve(m, ids[k], by_gid);
    if (h < 0) {
        if (counters && l == 0) atomicAdd(&counters[2], 1ull);
        return;
    }
    if (owner[h] != static_cast<long long>(k)) return;        // a later position updates the same vertex
    const int32_t s = m.slot[h];
    char *d = s >= 0 ? gpu_table + static_cast<int64_t>(s) * pitch : host_table + (-1 - static_cast<int64_t>(s)) * pitch;
    copy_row(rows + k * rows_pitch, d, row_bytes, l, lpr, vec16, es);
    // a copy of the host tier that was prefetched for the next epoch gets the new row as well
    if (s < 0 && staged_table)
        copy_row(rows + k * rows_pitch, staged_table + (-1 - static_cast<int64_t>(s)) * pitch, row_bytes, l, lpr, vec16, es);
    if (counters && l == 0) atomicAdd(&counters[s >= 0 ? 0 : 1], 1ull);
    if (l == 0) stamp[h] = epoch;
}

__global__ __launch_bounds__(256) void update_clear_kernel(MapView m, const int64_t *ids, int64_t n, int by_gid,
                                                           long long *owner) {
    const int64_t k = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (k >= n) return;
    const int64_t h = resolve(m, ids[k], by_gid);
    if (h >= 0) owner[h] = -1;
}

__global__ __launch_bounds__(256) void fill_i64_kernel(int64_t *p, int64_t n, int64_t v) {
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; i < n; i += static_cast<int64_t>(gridDim.x) * 256)
        p[i] = v;
}

// ---- stale list: ordered compaction in three steps (count per 1024-row block, scan of the counts, write)
constexpr int STALE_BLOCK = 1024;

__global__ __launch_bounds__(STALE_BLOCK) void stale_count_kernel(const int64_t *stamp, int64_t n, int64_t epoch_now,
                                                                   int64_t max_age, int64_t *counts, long long *oldest) {
    __shared__ int red[STALE_BLOCK];
    __shared__ long long lo[STALE_BLOCK];
    const int64_t h = static_cast<int64_t>(blockIdx.x) * STALE_BLOCK + threadIdx.x;
    const bool in = h < n;
    const int64_t st = in ? stamp[h] : epoch_now;
    red[threadIdx.x] = (in && epoch_now - st > max_age) ? 1 : 0;
    lo[threadIdx.x] = st;
    __syncthreads();
    for (int s = STALE_BLOCK / 2; s > 0; s >>= 1) {
        if (threadIdx.x < s) {
            red[threadIdx.x] += red[threadIdx.x + s];
            lo[threadIdx.x] = lo[threadIdx.x] < lo[threadIdx.x + s] ? lo[threadIdx.x] : lo[threadIdx.x + s];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        counts[blockIdx.x] = red[0];
        atomicMin(oldest, lo[0]);
    }
}

// counts[b] <- number of stale rows before block b; counts[nb] <- total.  One workgroup: every thread sums a
// contiguous run of counts, the run totals are scanned through LDS, then each thread writes its run's offsets.
__global__ __launch_bounds__(STALE_BLOCK) void stale_scan_kernel(int64_t *counts, int64_t nb) {
    __shared__ long long tot[STALE_BLOCK];
    const int64_t per = (nb + STALE_BLOCK - 1) / STALE_BLOCK;
    const int64_t lo = threadIdx.x * per, hi = lo + per < nb ? lo + per : nb;
    long long sum = 0;
    for (int64_t b = lo; b < hi; ++b) sum += counts[b];
    tot[threadIdx.x] = sum;
    __syncthreads();
    for (int off = 1; off < STALE_BLOCK; off <<= 1) {
        const long long v = threadIdx.x >= off ? tot[threadIdx.x - off] : 0;
        __syncthreads();
        tot[threadIdx.x] += v;
        __syncthreads();
    }
    long long run = tot[threadIdx.x] - sum;      // exclusive prefix of this thread's run
    for (int64_t b = lo; b < hi; ++b) {
        const int64_t c = counts[b];
        counts[b] = run;
        run += c;
    }
    if (threadIdx.x == STALE_BLOCK - 1) counts[nb] = tot[STALE_BLOCK - 1];
}

__global__ __launch_bounds__(STALE_BLOCK) void stale_write_kernel(const int64_t *stamp, int64_t n, int64_t epoch_now,
                                                                   int64_t max_age, const int64_t *counts, int64_t *ids_out) {
    __shared__ int pre[STALE_BLOCK];
    const int64_t h = static_cast<int64_t>(blockIdx.x) * STALE_BLOCK + threadIdx.x;
    const int flag = (h < n && epoch_now - stamp[h] > max_age) ? 1 : 0;
    pre[threadIdx.x] = flag;
    __syncthreads();
    for (int off = 1; off < STALE_BLOCK; off <<= 1) {          // inclusive prefix sum of the flags
        const int v = threadIdx.x >= off ? pre[threadIdx.x - off] : 0;
        __syncthreads();
        pre[threadIdx.x] += v;
        __syncthreads();
    }
    if (flag) ids_out[counts[blockIdx.x] + pre[threadIdx.x] - 1] = h;
}

__global__ void zero_counters_kernel(unsigned long long *c) {
    if (threadIdx.x < 4) c[threadIdx.x] = 0ull;
}

static int lanes_per_row(int row_bytes, int vec16, int es) {
    const int units = vec16 ? (row_bytes + 15) / 16 : (row_bytes + es - 1) / es;
    int lpr = 4;
    while (lpr < 64 && lpr < units) lpr <<= 1;
    return lpr;
}

struct CopyGeom {
    int row_bytes, lpr, vec16, es;
    int64_t out_pitch;
};

static int copy_geom(const capgnn_cache *c, int layer, const void *out, int64_t ld, const void *src_base, CopyGeom *g) {
    g->es = elem_bytes(c->dtype);
    g->row_bytes = c->dims[layer] * g->es;
    g->out_pitch = ld * g->es;
    if (ld < c->dims[layer]) CG_FAIL(CAPGNN_EINVAL, "halo_gather: ld=%lld smaller than the row width %d", (long long)ld, c->dims[layer]);
    g->vec16 = aligned16(out) && g->out_pitch % 16 == 0 && aligned16(src_base) && c->pitch[layer] % 16 == 0;
    g->lpr = lanes_per_row(g->row_bytes, g->vec16, g->es);
    return CAPGNN_OK;
}

static MapView view_dev(const capgnn_cache *c) {
    MapView m;
    m.n_halo = c->n_halo; m.slot = c->slot_d; m.hkeys = c->hkeys_d; m.hvals = c->hvals_d; m.hmask = c->hmask;
    return m;
}

static MapView view_host(const capgnn_cache *c) {
    MapView m;
    m.n_halo = c->n_halo; m.slot = c->slot_h.data();
    m.hkeys = c->hkeys_h.empty() ? nullptr : c->hkeys_h.data();
    m.hvals = c->hvals_h.empty() ? nullptr : c->hvals_h.data();
    m.hmask = c->hmask;
    return m;
}

constexpr unsigned HOST_READ_BLOCKS = 128;

static unsigned blocks_for(int64_t n, int lpr) {
    const int64_t rows_per_block = 4 * (64 / lpr);
    return static_cast<unsigned>((n + rows_per_block - 1) / rows_per_block);
}

static unsigned scatter_blocks_for(int64_t n, int lpr) {
    const int64_t rows_per_block = 4 * (64 / lpr) * SCATTER_ROWS;
    return static_cast<unsigned>((n + rows_per_block - 1) / rows_per_block);
}

// GPU-tier part of the full-batch gather of one layer, on `st`.
int gather_all_hits(const capgnn_cache *c, int layer, void *out, int64_t ld, hipStream_t st) {
    if (c->cap_gpu == 0) return CAPGNN_OK;
    CopyGeom g;
    const char *tab = c->gpu_tier + c->gpu_off[layer];
    CG_TRY(copy_geom(c, layer, out, ld, tab, &g));
    const TierRows a{tab, c->gpu_list_d, c->cap_gpu, scatter_blocks_for(c->cap_gpu, g.lpr)}, none{nullptr, nullptr, 0, 0};
    hipLaunchKernelGGL(scatter_tier_kernel, dim3(a.blocks), dim3(256), 0, st, a, none, c->pitch[layer],
                       static_cast<char *>(out), g.out_pitch, g.row_bytes, g.lpr, g.vec16, g.es);
    CG_HIP(hipGetLastError());
    return CAPGNN_OK;
}

// Both device-resident sources of one layer's halo rows in one launch: the GPU tier and the staged copy of the host
// tier (the caller has made `st` wait for that copy).
int gather_hits_and_staged(const capgnn_cache *c, int layer, void *out, int64_t ld, void *staging, hipStream_t st) {
    if (c->cap_gpu == 0) return scatter_staged(c, layer, out, ld, staging, st);
    if (c->n_host == 0) return gather_all_hits(c, layer, out, ld, st);
    if (!staging) CG_FAIL(CAPGNN_EINVAL, "halo_gather: staging area is NULL");
    const char *tab = c->gpu_tier + c->gpu_off[layer];
    const char *stab = static_cast<const char *>(staging) + c->host_off[layer];
    CopyGeom g, gs;
    CG_TRY(copy_geom(c, layer, out, ld, tab, &g));
    CG_TRY(copy_geom(c, layer, out, ld, stab, &gs));
    if (g.vec16 != gs.vec16 || g.lpr != gs.lpr) {       // differently aligned sources: one launch each
        CG_TRY(gather_all_hits(c, layer, out, ld, st));
        return scatter_staged(c, layer, out, ld, staging, st);
    }
    const TierRows a{tab, c->gpu_list_d, c->cap_gpu, scatter_blocks_for(c->cap_gpu, g.lpr)};
    const TierRows b{stab, c->host_list_d, c->n_host, scatter_blocks_for(c->n_host, g.lpr)};
    hipLaunchKernelGGL(scatter_tier_kernel, dim3(a.blocks + b.blocks), dim3(256), 0, st, a, b, c->pitch[layer],
                       static_cast<char *>(out), g.out_pitch, g.row_bytes, g.lpr, g.vec16, g.es);
    CG_HIP(hipGetLastError());
    return CAPGNN_OK;
}

// DMA of layer `layer`'s host tier into its slot of the staging area.
int stage_misses(const capgnn_cache *c, int layer, void *staging, hipStream_t st) {
    if (c->n_host == 0) return CAPGNN_OK;
    if (!staging) CG_FAIL(CAPGNN_EINVAL, "halo_gather: staging area is NULL");
    CG_HIP(hipMemcpyAsync(static_cast<char *>(staging) + c->host_off[layer], c->host_tier + c->host_off[layer],
                          static_cast<size_t>(c->n_host) * c->pitch[layer], hipMemcpyHostToDevice, st));
    return CAPGNN_OK;
}

static int scatter_host_rows(const capgnn_cache *c, int layer, const char *tab, bool pinned, void *out, int64_t ld,
                             hipStream_t st) {
    CopyGeom g;
    CG_TRY(copy_geom(c, layer, out, ld, tab, &g));
    // A kernel that reads pinned memory is bound by the host link, not by the CUs: a small grid keeps enough
    // requests in flight and leaves the compute units to the kernels of the main stream.
    unsigned blocks = scatter_blocks_for(c->n_host, g.lpr);
    if (pinned && blocks > HOST_READ_BLOCKS) blocks = HOST_READ_BLOCKS;
    const TierRows a{tab, c->host_list_d, c->n_host, blocks}, none{nullptr, nullptr, 0, 0};
    hipLaunchKernelGGL(scatter_tier_kernel, dim3(blocks), dim3(256), 0, st, a, none, c->pitch[layer],
                       static_cast<char *>(out), g.out_pitch, g.row_bytes, g.lpr, g.vec16, g.es);
    CG_HIP(hipGetLastError());
    return CAPGNN_OK;
}

// Scatter of a staged host tier into the halo rows it belongs to.
int scatter_staged(const capgnn_cache *c, int layer, void *out, int64_t ld, void *staging, hipStream_t st) {
    if (c->n_host == 0) return CAPGNN_OK;
    return scatter_host_rows(c, layer, static_cast<const char *>(staging) + c->host_off[layer], false, out, ld, st);
}

// Host-tier part of the full-batch gather of one layer, on `st`: either a kernel that reads pinned
// memory directly, or a DMA copy into `staging` followed by the same scatter from device memory.
int gather_all_misses(const capgnn_cache *c, int layer, void *out, int64_t ld, void *staging, hipStream_t st) {
    if (c->n_host == 0) return CAPGNN_OK;
    if (staging) {
        CG_TRY(stage_misses(c, layer, staging, st));
        return scatter_staged(c, layer, out, ld, staging, st);
    }
    return scatter_host_rows(c, layer, c->host_tier + c->host_off[layer], true, out, ld, st);
}

template <typename T>
static int dev_copy(capgnn_cache *c, const std::vector<T> &h, T **d) {
    void *p = nullptr;
    const size_t bytes = std::max<size_t>(h.size(), 1) * sizeof(T);
    if (hipMalloc(&p, bytes) != hipSuccess) CG_FAIL(CAPGNN_ENOMEM, "cache_build: hipMalloc of %zu bytes failed", bytes);
    c->dev_allocs.push_back(p);
    if (!h.empty()) CG_HIP(hipMemcpy(p, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice));
    *d = static_cast<T *>(p);
    return CAPGNN_OK;
}

}  // namespace capgnn

using namespace capgnn;

extern "C" int capgnn_cal_capacity(double mem_gb, double reserved_mb, const int32_t *dims, int n_layers,
                                   int elem_bytes_, int64_t n_candidates, int64_t *capacity_rows) {
    if (!dims || n_layers <= 0 || !capacity_rows || n_candidates < 0 || (elem_bytes_ != 4 && elem_bytes_ != 2))
        CG_FAIL(CAPGNN_EINVAL, "cal_capacity: bad argument");
    long double den = 0;
    for (int k = 0; k < n_layers; ++k) {
        if (dims[k] <= 0) CG_FAIL(CAPGNN_EINVAL, "cal_capacity: dims[%d] must be positive", k);
        den += static_cast<long double>(dims[k]) * elem_bytes_;
    }
    const long double num = (static_cast<long double>(mem_gb) * 1024.0L - static_cast<long double>(reserved_mb)) * 1048576.0L;
    int64_t rows = 0;
    if (num > 0) {
        long double q = floorl(num / den);
        while ((q + 1) * den <= num) q += 1;
        while (q * den > num) q -= 1;
        rows = q > 9.0e18L ? INT64_MAX : static_cast<int64_t>(q);
    }
    *capacity_rows = std::min<int64_t>(rows, n_candidates);
    return CAPGNN_OK;
}

static int64_t pitch_of(int dim, int dtype) { return static_cast<int64_t>(align_up(static_cast<size_t>(dim) * elem_bytes(dtype), 16)); }

extern "C" int capgnn_cache_sizes(int64_t n_halo, int64_t cap_gpu, const int32_t *dims, int n_layers, int dtype,
                                  size_t *gpu_bytes, size_t *host_bytes, size_t *staging_bytes) {
    if (n_halo < 0 || cap_gpu < 0 || !dims || n_layers <= 0 || (dtype != CAPGNN_F32 && dtype != CAPGNN_BF16))
        CG_FAIL(CAPGNN_EINVAL, "cache_sizes: bad argument");
    const int64_t k = std::min(cap_gpu, n_halo);
    size_t gb = 0, hb = 0;
    for (int l = 0; l < n_layers; ++l) {
        if (dims[l] <= 0) CG_FAIL(CAPGNN_EINVAL, "cache_sizes: dims[%d] must be positive", l);
        gb += align_up(static_cast<size_t>(k) * pitch_of(dims[l], dtype), 256);
        hb += align_up(static_cast<size_t>(n_halo - k) * pitch_of(dims[l], dtype), 256);
    }
    if (gpu_bytes) *gpu_bytes = gb;
    if (host_bytes) *host_bytes = hb;
    if (staging_bytes) *staging_bytes = hb;
    return CAPGNN_OK;
}

extern "C" int capgnn_cache_build(capgnn_cache **out, int64_t n_halo, const int64_t *gid, const int64_t *prio,
                                  int64_t cap_gpu, const int32_t *dims, int n_layers, int dtype, void *gpu_tier,
                                  void *host_tier, int map_kind, void *stream) {
    if (!out) CG_FAIL(CAPGNN_EINVAL, "cache_build: c is NULL");
    *out = nullptr;
    if (n_halo < 0 || n_halo >= (int64_t(1) << 31) - 1 || cap_gpu < 0 || !dims || n_layers <= 0 ||
        (dtype != CAPGNN_F32 && dtype != CAPGNN_BF16) || (map_kind != CAPGNN_MAP_DIRECT && map_kind != CAPGNN_MAP_HASH))
        CG_FAIL(CAPGNN_EINVAL, "cache_build: bad argument");
    if (n_halo > 0 && (!gid || !prio)) CG_FAIL(CAPGNN_EINVAL, "cache_build: gid/prio is NULL");
    const int64_t k = std::min(cap_gpu, n_halo);
    if (k > 0 && !gpu_tier) CG_FAIL(CAPGNN_EINVAL, "cache_build: gpu_tier is NULL");
    if (n_halo - k > 0 && !host_tier) CG_FAIL(CAPGNN_EINVAL, "cache_build: host_tier is NULL");
    if ((reinterpret_cast<uintptr_t>(gpu_tier) | reinterpret_cast<uintptr_t>(host_tier)) & 255u)
        CG_FAIL(CAPGNN_EINVAL, "cache_build: tiers must be 256-byte aligned");
    for (int l = 0; l < n_layers; ++l)
        if (dims[l] <= 0) CG_FAIL(CAPGNN_EINVAL, "cache_build: dims[%d] must be positive", l);
    {
        std::vector<int64_t> s(gid, gid + n_halo);
        std::sort(s.begin(), s.end());
        if (std::adjacent_find(s.begin(), s.end()) != s.end()) CG_FAIL(CAPGNN_EINVAL, "cache_build: duplicate global id");
    }
    capgnn_cache *c = new (std::nothrow) capgnn_cache();
    if (!c) CG_FAIL(CAPGNN_ENOMEM, "cache_build: out of host memory");
    auto fail = [&](int rc) { capgnn_cache_destroy(c); return rc; };
    c->n_halo = n_halo; c->cap_gpu = k; c->n_host = n_halo - k; c->n_layers = n_layers; c->dtype = dtype;
    c->map_kind = map_kind;
    c->dims.assign(dims, dims + n_layers);
    c->gpu_tier = static_cast<char *>(gpu_tier);
    c->host_tier = static_cast<char *>(host_tier);
    size_t go = 0, ho = 0;
    for (int l = 0; l < n_layers; ++l) {
        c->pitch.push_back(pitch_of(dims[l], dtype));
        c->gpu_off.push_back(go);
        c->host_off.push_back(ho);
        go += align_up(static_cast<size_t>(k) * c->pitch[l], 256);
        ho += align_up(static_cast<size_t>(c->n_host) * c->pitch[l], 256);
    }
    // placement: rank by (priority descending, global id ascending)
    std::vector<int32_t> rank(n_halo);
    std::iota(rank.begin(), rank.end(), 0);
    std::sort(rank.begin(), rank.end(), [&](int32_t a, int32_t b) {
        if (prio[a] != prio[b]) return prio[a] > prio[b];
        return gid[a] < gid[b];
    });
    std::vector<uint8_t> on_gpu(n_halo, 0);
    for (int64_t r = 0; r < k; ++r) on_gpu[rank[r]] = 1;
    c->slot_h.resize(n_halo);
    c->gid_h.assign(gid, gid + n_halo);
    std::vector<int32_t> gpu_list, host_list;
    gpu_list.reserve(k);
    host_list.reserve(n_halo - k);
    for (int64_t h = 0; h < n_halo; ++h) {
        if (on_gpu[h]) { c->slot_h[h] = static_cast<int32_t>(gpu_list.size()); gpu_list.push_back(static_cast<int32_t>(h)); }
        else { c->slot_h[h] = -1 - static_cast<int32_t>(host_list.size()); host_list.push_back(static_cast<int32_t>(h)); }
    }
    if (map_kind == CAPGNN_MAP_HASH) {
        uint64_t cap = 16;
        while (cap < static_cast<uint64_t>(n_halo) * 2) cap <<= 1;
        c->hmask = cap - 1;
        c->hkeys_h.assign(cap, 0);
        c->hvals_h.assign(cap, -1);
        for (int64_t h = 0; h < n_halo; ++h) {
            uint64_t p = mix64(static_cast<uint64_t>(gid[h])) & c->hmask;
            while (c->hvals_h[p] >= 0) p = (p + 1) & c->hmask;
            c->hkeys_h[p] = gid[h];
            c->hvals_h[p] = static_cast<int32_t>(h);
        }
    }
    int rc;
    if ((rc = dev_copy(c, c->slot_h, &c->slot_d))) return fail(rc);
    if ((rc = dev_copy(c, gpu_list, &c->gpu_list_d))) return fail(rc);
    if ((rc = dev_copy(c, host_list, &c->host_list_d))) return fail(rc);
    if (map_kind == CAPGNN_MAP_HASH) {
        if ((rc = dev_copy(c, c->hkeys_h, &c->hkeys_d))) return fail(rc);
        if ((rc = dev_copy(c, c->hvals_h, &c->hvals_d))) return fail(rc);
    }
    std::vector<int64_t> zeros(4, 0);
    if ((rc = dev_copy(c, zeros, &c->counters_d))) return fail(rc);
    {
        std::vector<int64_t> stamps(static_cast<size_t>(n_layers) * n_halo, 0);
        std::vector<long long> owners(n_halo, -1);
        std::vector<int64_t> scan(n_halo / STALE_BLOCK + 3, 0);
        if ((rc = dev_copy(c, stamps, &c->stamp_d))) return fail(rc);
        if ((rc = dev_copy(c, owners, &c->owner_d))) return fail(rc);
        if ((rc = dev_copy(c, scan, &c->scan_d))) return fail(rc);
    }
    if (hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming) != hipSuccess) {
        set_error("cache_build: hipEventCreate failed");
        return fail(CAPGNN_EHIP);
    }
    c->ev_layer.assign(n_layers, nullptr);
    c->ev_consumed.assign(n_layers, nullptr);
    c->staged_valid.assign(n_layers, 0);
    for (int l = 0; l < n_layers; ++l)
        if (hipEventCreateWithFlags(&c->ev_layer[l], hipEventDisableTiming) != hipSuccess ||
            hipEventCreateWithFlags(&c->ev_consumed[l], hipEventDisableTiming) != hipSuccess) {
            set_error("cache_build: hipEventCreate failed");
            return fail(CAPGNN_EHIP);
        }
    if (hipStreamSynchronize(static_cast<hipStream_t>(stream)) != hipSuccess) {
        set_error("cache_build: stream synchronisation failed");
        return fail(CAPGNN_EHIP);
    }
    *out = c;
    return CAPGNN_OK;
}

extern "C" int capgnn_cache_destroy(capgnn_cache *c) {
    if (!c) return CAPGNN_OK;
    if (c->last_side) (void)hipStreamSynchronize(c->last_side);   // a prefetch may still be reading the host tier
    for (void *p : c->dev_allocs) (void)hipFree(p);
    if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
    if (c->ev_join) (void)hipEventDestroy(c->ev_join);
    for (hipEvent_t e : c->ev_layer) if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : c->ev_consumed) if (e) (void)hipEventDestroy(e);
    delete c;
    return CAPGNN_OK;
}

extern "C" int capgnn_cache_set_miss_mode(capgnn_cache *c, int mode) {
    if (!c || mode < CAPGNN_MISS_ZEROCOPY || mode > CAPGNN_MISS_PIPELINED) CG_FAIL(CAPGNN_EINVAL, "cache_set_miss_mode: bad argument");
    if (c->last_side) CG_HIP(hipStreamSynchronize(c->last_side));
    c->miss_mode = mode;
    std::fill(c->staged_valid.begin(), c->staged_valid.end(), 0);
    c->staged_base = nullptr;       // the workspace that held the prefetched copies may go away now
    return CAPGNN_OK;
}

extern "C" int capgnn_cache_fill(capgnn_cache *c, int layer, const void *rows, int64_t ld, void *stream) {
    if (!c || layer < 0 || layer >= c->n_layers) CG_FAIL(CAPGNN_EINVAL, "cache_fill: bad cache or layer");
    if (c->n_halo == 0) return CAPGNN_OK;
    if (!rows || ld < c->dims[layer]) CG_FAIL(CAPGNN_EINVAL, "cache_fill: rows is NULL or ld too small");
    if (c->last_side) CG_HIP(hipStreamSynchronize(c->last_side));   // a prefetch may be reading the host tier
    const int es = elem_bytes(c->dtype);
    const size_t rb = static_cast<size_t>(c->dims[layer]) * es;
    const int64_t pitch = c->pitch[layer];
    const char *src = static_cast<const char *>(rows);
    std::vector<char> pack(static_cast<size_t>(c->cap_gpu) * pitch, 0);
    char *host_tab = c->host_tier + c->host_off[layer];
    for (int64_t h = 0; h < c->n_halo; ++h) {
        const int32_t s = c->slot_h[h];
        char *dst = s >= 0 ? pack.data() + static_cast<size_t>(s) * pitch : host_tab + static_cast<size_t>(-1 - s) * pitch;
        std::memcpy(dst, src + static_cast<size_t>(h) * ld * es, rb);
        if (static_cast<size_t>(pitch) > rb) std::memset(dst + rb, 0, pitch - rb);
    }
    CG_HIP(hipStreamSynchronize(static_cast<hipStream_t>(stream)));
    if (c->cap_gpu > 0)
        CG_HIP(hipMemcpy(c->gpu_tier + c->gpu_off[layer], pack.data(), pack.size(), hipMemcpyHostToDevice));
    c->staged_valid[layer] = 0;      // rows prefetched for the next epoch are out of date now
    hipLaunchKernelGGL(fill_i64_kernel, dim3(256), dim3(256), 0, static_cast<hipStream_t>(stream),
                       c->stamp_d + static_cast<size_t>(layer) * c->n_halo, c->n_halo, int64_t(0));
    CG_HIP(hipGetLastError());
    CG_HIP(hipStreamSynchronize(static_cast<hipStream_t>(stream)));
    CG_HIP(hipDeviceSynchronize());   // setup call: the tables and stamps are in place for work on any stream
    return CAPGNN_OK;
}

extern "C" int capgnn_cache_query(const capgnn_cache *c, const int64_t *ids, int64_t n, int by_gid, int8_t *tier,
                                  int64_t *slot) {
    if (!c || n < 0 || (n > 0 && (!ids || !tier || !slot))) CG_FAIL(CAPGNN_EINVAL, "cache_query: bad argument");
    if (by_gid && c->map_kind != CAPGNN_MAP_HASH) CG_FAIL(CAPGNN_EINVAL, "cache_query: by_gid needs a cache built with MAP_HASH");
    const MapView m = view_host(c);
    int64_t absent = 0;
    for (int64_t k = 0; k < n; ++k) {
        const int64_t h = resolve(m, ids[k], by_gid);
        if (h < 0) { tier[k] = -1; slot[k] = -1; ++absent; continue; }
        const int32_t s = c->slot_h[h];
        tier[k] = s >= 0 ? 0 : 1;
        slot[k] = s >= 0 ? s : -1 - static_cast<int64_t>(s);
    }
    if (absent) CG_FAIL(CAPGNN_ENOTFOUND, "cache_query: %lld ids are in neither tier", (long long)absent);
    return CAPGNN_OK;
}

extern "C" int capgnn_cache_lookup(const capgnn_cache *c, const int64_t *ids, int64_t n, int by_gid, int8_t *tier,
                                   int64_t *slot, void *stream) {
    if (!c || n < 0 || (n > 0 && (!ids || !tier || !slot))) CG_FAIL(CAPGNN_EINVAL, "cache_lookup: bad argument");
    if (by_gid && c->map_kind != CAPGNN_MAP_HASH) CG_FAIL(CAPGNN_EINVAL, "cache_lookup: by_gid needs a cache built with MAP_HASH");
    if (n == 0) return CAPGNN_OK;
    hipLaunchKernelGGL(lookup_kernel, dim3(static_cast<unsigned>((n + 255) / 256)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), view_dev(c), ids, n, by_gid, tier, slot);
    CG_HIP(hipGetLastError());
    return CAPGNN_OK;
}

extern "C" int capgnn_halo_gather(capgnn_cache *c, int layer, const int64_t *ids, int64_t n, int by_gid, void *out,
                                  int64_t ld, void *stream, void *side_stream, void *staging,
                                  capgnn_gather_stats *stats) {
    if (!c || layer < 0 || layer >= c->n_layers) CG_FAIL(CAPGNN_EINVAL, "halo_gather: bad cache or layer");
    if (n < 0) CG_FAIL(CAPGNN_EINVAL, "halo_gather: n < 0");
    if (by_gid && c->map_kind != CAPGNN_MAP_HASH) CG_FAIL(CAPGNN_EINVAL, "halo_gather: by_gid needs a cache built with MAP_HASH");
    if (!ids && n != c->n_halo) CG_FAIL(CAPGNN_EINVAL, "halo_gather: ids == NULL needs n == n_halo");
    if (stats) stats->hits = stats->misses = stats->absent = 0;
    if (n == 0) return CAPGNN_OK;
    if (!out) CG_FAIL(CAPGNN_EINVAL, "halo_gather: out is NULL");
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipStream_t side = side_stream ? static_cast<hipStream_t>(side_stream) : st;
    const bool forked = side != st;

    if (!ids) {
        const bool has_miss = c->n_host > 0;
        if (forked && has_miss) {
            CG_HIP(hipEventRecord(c->ev_fork, st));
            CG_HIP(hipStreamWaitEvent(side, c->ev_fork, 0));
        }
        if (has_miss) CG_TRY(gather_all_misses(c, layer, out, ld, staging, side));
        CG_TRY(gather_all_hits(c, layer, out, ld, st));
        if (forked && has_miss) {
            CG_HIP(hipEventRecord(c->ev_join, side));
            CG_HIP(hipStreamWaitEvent(st, c->ev_join, 0));
        }
        if (stats) {
            CG_HIP(hipStreamSynchronize(st));
            stats->hits = c->cap_gpu;
            stats->misses = c->n_host;
        }
        return CAPGNN_OK;
    }

    CopyGeom g;
    const char *gtab = c->gpu_tier + c->gpu_off[layer];
    const char *htab = c->host_tier + c->host_off[layer];
    CG_TRY(copy_geom(c, layer, out, ld, gtab, &g));
    if (!(aligned16(htab))) g.vec16 = 0;
    unsigned long long *ctr = stats ? reinterpret_cast<unsigned long long *>(c->counters_d) : nullptr;
    if (ctr) hipLaunchKernelGGL(zero_counters_kernel, dim3(1), dim3(64), 0, st, ctr);
    const unsigned blocks = blocks_for(n, g.lpr);
    const MapView m = view_dev(c);
    if (forked && c->n_host > 0) {
        CG_HIP(hipEventRecord(c->ev_fork, st));
        CG_HIP(hipStreamWaitEvent(side, c->ev_fork, 0));
        hipLaunchKernelGGL(gather_ids_kernel, dim3(blocks), dim3(256), 0, side, m, ids, n, by_gid, gtab, htab,
                           c->pitch[layer], 2, static_cast<char *>(out), g.out_pitch, g.row_bytes, g.lpr, g.vec16, g.es, ctr);
        hipLaunchKernelGGL(gather_ids_kernel, dim3(blocks), dim3(256), 0, st, m, ids, n, by_gid, gtab, htab,
                           c->pitch[layer], 1, static_cast<char *>(out), g.out_pitch, g.row_bytes, g.lpr, g.vec16, g.es, ctr);
        CG_HIP(hipEventRecord(c->ev_join, side));
        CG_HIP(hipStreamWaitEvent(st, c->ev_join, 0));
    } else {
        hipLaunchKernelGGL(gather_ids_kernel, dim3(blocks), dim3(256), 0, st, m, ids, n, by_gid, gtab, htab,
                           c->pitch[layer], 3, static_cast<char *>(out), g.out_pitch, g.row_bytes, g.lpr, g.vec16, g.es, ctr);
    }
    CG_HIP(hipGetLastError());
    if (stats) {
        unsigned long long h[4] = {0, 0, 0, 0};
        CG_HIP(hipMemcpyAsync(h, ctr, sizeof(h), hipMemcpyDeviceToHost, st));
        CG_HIP(hipStreamSynchronize(st));
        stats->hits = static_cast<int64_t>(h[0]);
        stats->misses = static_cast<int64_t>(h[1]);
        stats->absent = static_cast<int64_t>(h[2]);
        if (h[2]) CG_FAIL(CAPGNN_ENOTFOUND, "halo_gather: %llu ids are in neither tier", h[2]);
    }
    return CAPGNN_OK;
}

extern "C" int capgnn_cache_update(capgnn_cache *c, int layer, const int64_t *ids, int64_t n, int by_gid,
                                   const void *rows, int64_t ld, int64_t epoch, void *stream,
                                   capgnn_gather_stats *stats) {
    if (!c || layer < 0 || layer >= c->n_layers) CG_FAIL(CAPGNN_EINVAL, "cache_update: bad cache or layer");
    if (n < 0) CG_FAIL(CAPGNN_EINVAL, "cache_update: n < 0");
    if (by_gid && c->map_kind != CAPGNN_MAP_HASH) CG_FAIL(CAPGNN_EINVAL, "cache_update: by_gid needs a cache built with MAP_HASH");
    if (stats) stats->hits = stats->misses = stats->absent = 0;
    if (n == 0 || c->n_halo == 0) return CAPGNN_OK;
    if (!ids || !rows) CG_FAIL(CAPGNN_EINVAL, "cache_update: ids or rows is NULL");
    if (ld < c->dims[layer]) CG_FAIL(CAPGNN_EINVAL, "cache_update: ld=%lld smaller than the row width %d", (long long)ld, c->dims[layer]);
    hipStream_t st = static_cast<hipStream_t>(stream);
    // a prefetch of the previous epoch may still be reading the host tier: let it finish.  Its copy stays valid: the
    // kernel writes every host-tier row it updates into that copy too, so the next epoch neither sees an old row nor has
    // to fetch the table again (GPU-tier rows never were in the copy).
    if (c->last_side) CG_HIP(hipStreamSynchronize(c->last_side));
    const int es = elem_bytes(c->dtype);
    char *gtab = c->gpu_tier + c->gpu_off[layer];
    char *htab = c->host_tier + c->host_off[layer];
    char *stab = (c->n_host > 0 && c->staged_valid[layer] && c->staged_base)
                     ? static_cast<char *>(c->staged_base) + c->host_off[layer] : nullptr;
    const int row_bytes = c->dims[layer] * es;
    const int64_t rows_pitch = ld * es;
    const int vec16 = aligned16(rows) && rows_pitch % 16 == 0 && aligned16(gtab) && aligned16(htab) && (!stab || aligned16(stab)) &&
                      c->pitch[layer] % 16 == 0;
    const int lpr = lanes_per_row(row_bytes, vec16, es);
    const MapView m = view_dev(c);
    unsigned long long *ctr = stats ? reinterpret_cast<unsigned long long *>(c->counters_d) : nullptr;
    if (ctr) hipLaunchKernelGGL(zero_counters_kernel, dim3(1), dim3(64), 0, st, ctr);
    const unsigned b1 = static_cast<unsigned>((n + 255) / 256);
    hipLaunchKernelGGL(update_owner_kernel, dim3(b1), dim3(256), 0, st, m, ids, n, by_gid, c->owner_d);
    hipLaunchKernelGGL(update_rows_kernel, dim3(blocks_for(n, lpr)), dim3(256), 0, st, m, ids, n, by_gid,
                       static_cast<const char *>(rows), rows_pitch, gtab, htab, stab, c->pitch[layer], row_bytes, lpr, vec16, es,
                       c->owner_d, c->stamp_d + static_cast<size_t>(layer) * c->n_halo, epoch, ctr);
    hipLaunchKernelGGL(update_clear_kernel, dim3(b1), dim3(256), 0, st, m, ids, n, by_gid, c->owner_d);
    CG_HIP(hipGetLastError());
    if (stats) {
        unsigned long long h[4] = {0, 0, 0, 0};
        CG_HIP(hipMemcpyAsync(h, ctr, sizeof(h), hipMemcpyDeviceToHost, st));
        CG_HIP(hipStreamSynchronize(st));
        stats->hits = static_cast<int64_t>(h[0]);
        stats->misses = static_cast<int64_t>(h[1]);
        stats->absent = static_cast<int64_t>(h[2]);
    }
    return CAPGNN_OK;
}

extern "C" int capgnn_cache_stale(capgnn_cache *c, int layer, int64_t epoch_now, int64_t max_age, int64_t *ids_out,
                                  int64_t *n_out, int64_t *oldest, void *stream) {
    if (!c || layer < 0 || layer >= c->n_layers || !n_out) CG_FAIL(CAPGNN_EINVAL, "cache_stale: bad argument");
    *n_out = 0;
    if (oldest) *oldest = epoch_now;
    if (c->n_halo == 0) return CAPGNN_OK;
    if (!ids_out) CG_FAIL(CAPGNN_EINVAL, "cache_stale: ids_out is NULL");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t nb = (c->n_halo + STALE_BLOCK - 1) / STALE_BLOCK;
    const int64_t *stamp = c->stamp_d + static_cast<size_t>(layer) * c->n_halo;
    long long *lo = reinterpret_cast<long long *>(c->scan_d + nb + 1);
    hipLaunchKernelGGL(fill_i64_kernel, dim3(1), dim3(256), 0, st, c->scan_d + nb + 1, int64_t(1), epoch_now);
    hipLaunchKernelGGL(stale_count_kernel, dim3(static_cast<unsigned>(nb)), dim3(STALE_BLOCK), 0, st, stamp, c->n_halo,
                       epoch_now, max_age, c->scan_d, lo);
    hipLaunchKernelGGL(stale_scan_kernel, dim3(1), dim3(STALE_BLOCK), 0, st, c->scan_d, nb);
    hipLaunchKernelGGL(stale_write_kernel, dim3(static_cast<unsigned>(nb)), dim3(STALE_BLOCK), 0, st, stamp, c->n_halo,
                       epoch_now, max_age, c->scan_d, ids_out);
    CG_HIP(hipGetLastError());
    int64_t tail[2] = {0, 0};
    CG_HIP(hipMemcpyAsync(tail, c->scan_d + nb, sizeof(tail), hipMemcpyDeviceToHost, st));
    CG_HIP(hipStreamSynchronize(st));
    *n_out = tail[0];
    if (oldest) *oldest = tail[1];
    return CAPGNN_OK;
}
