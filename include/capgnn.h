/*
 * capgnn.h - C ABI of the MI355X-native partition-local layer step of cache-assisted
 * full-batch GNN training (CaPGNN, arxiv 2508.13716).
 *
 * One GPU's share of the method: the halo rows of each layer input are taken from a
 * two-tier cache (GPU memory = local cache, pinned host memory = global cache; section
 * "Joint Adaptive Caching Algorithm"), then a GCN or GraphSAGE-mean layer runs on the
 * partition's local+halo graph (aggregate, combine; Eq. 1 and the forward rule in the proof
 * of Lemma 2), followed by the backward pass (the chain rule behind Lemma 3).
 *
 * Conventions
 *   - Every call returns an int: 0 = CAPGNN_OK, < 0 = error.  Nothing is printed, nothing
 *     aborts.  capgnn_last_error() gives a text for the most recent failure on this thread.
 *   - "device" pointers are HIP device memory, "host" pointers are ordinary host memory,
 *     "pinned" pointers are page-locked host memory that the GPU can read (hipHostMalloc).
 *   - The caller owns every feature / activation / gradient / weight / cache-tier buffer.
 *     The library owns only its opaque handles and the index structures inside them
 *     (CSR/CSC copies, slot maps), which it allocates at create/build time and frees at destroy.
 *   - Device work is enqueued on the caller's stream (void* = hipStream_t, NULL = default
 *     stream) and the call returns without synchronising unless the call says otherwise.
 *   - Matrices are row-major with an explicit leading dimension `ld` counted in ELEMENTS;
 *     a buffer with n rows must hold n*ld elements.  dtype selects the storage type of
 *     features/activations: CAPGNN_F32 (float) or CAPGNN_BF16 (bfloat16 bits, fp32 accumulate,
 *     round-to-nearest-even on store).  Scales, biases and weight gradients are always float.
 *   - Scratch memory is caller-provided: ask *_workspace_bytes(), pass (ws, ws_bytes).
 *     ws must be 256-byte aligned device memory.
 *   - Handles are not thread-safe; distinct handles are independent.
 */
#ifndef CAPGNN_H
#define CAPGNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CAPGNN_OK            0
#define CAPGNN_EINVAL       (-1)  /* bad argument (shape, alignment, NULL, range)         */
#define CAPGNN_ENOMEM       (-2)  /* host or device allocation failed / workspace too small */
#define CAPGNN_EHIP         (-3)  /* a HIP runtime call failed (text in capgnn_last_error) */
#define CAPGNN_ENOTFOUND    (-4)  /* a requested id is in neither cache tier              */
#define CAPGNN_EUNSUPPORTED (-5)  /* valid request this build does not implement          */

#define CAPGNN_F32   0
#define CAPGNN_BF16  1

#define CAPGNN_GCN        0
#define CAPGNN_SAGE_MEAN  1

#define CAPGNN_ACT_NONE 0
#define CAPGNN_ACT_RELU 1

#define CAPGNN_ORDER_AUTO   0   /* library picks the cheaper association of A_hat X W          */
#define CAPGNN_AGG_FIRST    1   /* (A_hat X) W : SpMM at f_in, GEMM over local rows            */
#define CAPGNN_XFORM_FIRST  2   /* A_hat (X W) : GEMM over all columns, SpMM at f_out          */

#define CAPGNN_MAP_DIRECT 0     /* ids are halo-local indices 0..n_halo-1                     */
#define CAPGNN_MAP_HASH   1     /* additionally build a hash table over the 64-bit global ids */

#define CAPGNN_NORM_SYM   0     /* r_i = d_i^-1/2, c_j = d_j^-1/2 (symmetric normalisation)    */
#define CAPGNN_NORM_MEAN  1     /* r_i = 1/d_i (0 for empty rows), c_j = 1 (mean aggregator)   */

#define CAPGNN_GRAPH_SYMMETRIC 1u  /* n_halo == 0 and A_hat^T == A_hat: backward reuses the CSR */

#define CAPGNN_MISS_ZEROCOPY  0  /* host-tier rows are read by a kernel straight from pinned memory */
#define CAPGNN_MISS_STAGED    1  /* host tier is DMA-copied into a device staging area, then scattered (default) */
#define CAPGNN_MISS_PIPELINED 2  /* as STAGED, and capgnn_epoch starts the copy for the NEXT epoch as soon as this
                                    epoch has consumed a layer's staging area (the prefetch queue of the section
                                    "Pipeline Design": transfers overlap computation across iterations) */

typedef struct capgnn_graph capgnn_graph;
typedef struct capgnn_cache capgnn_cache;

const char *capgnn_last_error(void);
int capgnn_version(void);

/* ------------------------------------------------------------------------------------------
 * Graph: the partition's local+halo graph.  Rows = local (inner) vertices, columns = local
 * vertices [0,n_loc) followed by halo vertices [n_loc, n_loc+n_halo) (section "Graph
 * Partition": halo vertices are the remote endpoints of cut edges; they have no rows).
 * A_hat[i,j] = row_scale[i] * A[i,j] * col_scale[j], A[i,j] = sum of edge_val over stored
 * entries (i,j) (1 each when edge_val is NULL).
 * ---------------------------------------------------------------------------------------- */

/* Host helper: the default scales.  CAPGNN_NORM_SYM follows the notation table's "adjacency
 * matrix after symmetric normalization": d_i = stored entries of row i (a self loop, if the
 * caller wants one, must be among them), clamped to >= 1; local column j uses row j's d;
 * halo column h uses halo_degree[h] (its degree in the whole graph, host, may be NULL = 1).
 * CAPGNN_NORM_MEAN is the mean aggregator of GraphSAGE (Eq. 1 with AGGREGATE = mean).
 * rowptr: host int64[n_loc+1]; outputs: host float[n_loc], float[n_loc+n_halo].  No GPU work. */
int capgnn_norm_scales(int kind, int64_t n_loc, int64_t n_halo, const int64_t *rowptr,
                       const int64_t *halo_degree, float *row_scale, float *col_scale);

/* Host helper: the operator of a GIN layer's aggregation, (1 + eps) x_i + sum_{j in N(i)} x_j (the paper's
 * convergence analysis names GIN among the covered architectures: neighbour aggregation, a linear transform, a
 * Lipschitz nonlinearity).  Output CSR = the input's entries with value 1 plus one diagonal entry of value 1 + eps
 * appended to every row: rowptr_out host int64[n_loc+1], col_out host int32[nnz+n_loc], val_out host float[nnz+n_loc].
 * Pass it to capgnn_graph_create with edge_val = val_out and no scales; a CAPGNN_GCN layer on that graph is a GIN
 * layer with a one-layer update function.  No GPU work. */
int capgnn_gin_operator(int64_t n_loc, int64_t n_halo, const int64_t *rowptr, const int32_t *col, float eps,
                        int64_t *rowptr_out, int32_t *col_out, float *val_out);

/* Uploads the CSR, builds the CSC (= CSR of A_hat^T) and the degree-ordered work lists.
 * rowptr: host int64[n_loc+1], rowptr[0]==0, non-decreasing; col: host int32[nnz], each in
 * [0, n_loc+n_halo); nnz < 2^31.  row_scale/col_scale: host float arrays or NULL (= 1).
 * edge_val: host float[nnz] or NULL.  Synchronises `stream` before returning (setup call).
 * Errors: EINVAL on malformed CSR, ENOMEM, EHIP. */
int capgnn_graph_create(capgnn_graph **g, int64_t n_loc, int64_t n_halo,
                        const int64_t *rowptr, const int32_t *col,
                        const float *row_scale, const float *col_scale, const float *edge_val,
                        uint32_t flags, void *stream);
int capgnn_graph_destroy(capgnn_graph *g);

/* ------------------------------------------------------------------------------------------
 * Aggregation (the SpMM term of RAPA's cost model, Eq. 4; the `aggregation` stage of the evaluation's
 * stage breakdown).
 * ---------------------------------------------------------------------------------------- */

/* Y[i,0:F] = row_scale[i] * sum_{e in row i} edge_val[e]*col_scale[col e] * X[col e, 0:F], i < n_loc.
 * X: device [n_cols x ldx], Y: device [n_loc x ldy], both of `dtype`; accumulation in fp32.
 * Fast path needs 16-byte aligned bases and row pitches; other layouts run a scalar path. */
size_t capgnn_spmm_workspace_bytes(const capgnn_graph *g, int F, int dtype);
int capgnn_spmm_fwd(const capgnn_graph *g, const void *X, int64_t ldx, void *Y, int64_t ldy,
                    int F, int dtype, void *ws, size_t ws_bytes, void *stream);

/* dX[j,0:F] = col_scale[j] * sum_{e: col e = j} edge_val[e]*row_scale[row e] * dY[row e, 0:F], j < n_cols
 * (= A_hat^T dY; the product the backward recursion of Lemma 3 needs).  Atomic-free: runs over the
 * CSC built at create time.  dY: device [n_loc x lddy]; dX: device [n_cols x lddx]. */
int capgnn_spmm_bwd(const capgnn_graph *g, const void *dY, int64_t lddy, void *dX, int64_t lddx,
                    int F, int dtype, void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------------------------
 * Joint cache (section "Joint Adaptive Caching Algorithm"): which halo vertices live in GPU
 * memory, which in pinned host memory, and the lookup / gather that fills a layer input.
 * ---------------------------------------------------------------------------------------- */

/* Adaptive cache capacity, Alg. 1 (cal_capacity): rows = min(floor(((mem_gb*1024 - reserved_mb)
 * * 1024^2) / sum_k(dims[k]*elem_bytes)), n_candidates), never negative.  The paper fixes
 * elem_bytes = 4 (fp32 rows); 2 is this library's extension for bf16 tables.  Host only. */
int capgnn_cal_capacity(double mem_gb, double reserved_mb, const int32_t *dims, int n_layers,
                        int elem_bytes, int64_t n_candidates, int64_t *capacity_rows);

/* Bytes the caller must provide for the two tiers (all layers) and, for CAPGNN_MISS_STAGED,
 * for the device staging area.  Row pitch of layer l's table = dims[l] rounded up to 16 bytes. */
int capgnn_cache_sizes(int64_t n_halo, int64_t cap_gpu, const int32_t *dims, int n_layers, int dtype,
                       size_t *gpu_bytes, size_t *host_bytes, size_t *staging_bytes);

/* Placement: halo vertices ranked by (prio descending, gid ascending); the first min(cap_gpu,n_halo)
 * go to the GPU tier, the rest to the host tier (priority = vertex overlap ratio, Eq. 2, or any
 * other importance the caller supplies).  gid, prio: host int64[n_halo], gid unique.
 * dims[l] = width of the rows cached for layer l's input (Alg. 1's f_dim).  gpu_tier: device,
 * host_tier: pinned, both caller-owned and at least capgnn_cache_sizes() bytes, 256-byte aligned.
 * Builds the id -> (tier, slot) map (direct array; plus a hash table over gid for MAP_HASH).
 * Synchronises `stream`.  Errors: EINVAL (duplicate gid, bad sizes), ENOMEM, EHIP. */
int capgnn_cache_build(capgnn_cache **c, int64_t n_halo, const int64_t *gid, const int64_t *prio,
                       int64_t cap_gpu, const int32_t *dims, int n_layers, int dtype,
                       void *gpu_tier, void *host_tier, int map_kind, void *stream);
int capgnn_cache_destroy(capgnn_cache *c);

/* How capgnn_epoch moves host-tier rows: CAPGNN_MISS_ZEROCOPY, CAPGNN_MISS_STAGED (default) or
 * CAPGNN_MISS_PIPELINED (for the last two capgnn_epoch_workspace_bytes() includes the staging area).
 * CAPGNN_MISS_PIPELINED keeps state between calls of capgnn_epoch: the staging area inside `ws` holds the
 * host-tier rows prefetched for the next call, so consecutive calls must pass the same ws (a different ws,
 * capgnn_cache_fill or a mode change make the next call fetch afresh), a side stream must be given, and copies
 * into ws may still be in flight on the side stream after capgnn_epoch returns: synchronise that stream (or the
 * device) before freeing or reusing ws, the tiers or the cache.  The rows an epoch consumes are the host
 * tier's contents at the time of the previous call (or of this call, for the first), plus every row that
 * capgnn_cache_update has written since.  The library cannot see other writes: a caller that writes the pinned tier
 * itself, or lets anything else use ws between two calls, calls capgnn_cache_set_miss_mode again (any mode), which
 * drops the prefetched copies. */
int capgnn_cache_set_miss_mode(capgnn_cache *c, int mode);

/* Loads layer `layer`'s logical table (host, [n_halo x ld], halo-local row order) into both tiers.
 * Synchronous (setup call): waits for `stream` and for a prefetch the last capgnn_epoch left in flight. */
int capgnn_cache_fill(capgnn_cache *c, int layer, const void *rows, int64_t ld, void *stream);

/* check_cache on the host (for tests and planning): ids are halo-local indices, or global ids when
 * by_gid != 0 (needs MAP_HASH).  tier[k] = 0 GPU, 1 host, -1 absent; slot[k] = row inside that tier
 * (-1 if absent).  All arrays host.  Returns ENOTFOUND if any id is absent (outputs still complete). */
int capgnn_cache_query(const capgnn_cache *c, const int64_t *ids, int64_t n, int by_gid,
                       int8_t *tier, int64_t *slot);

/* check_cache on the GPU: same result, ids / tier / slot are device arrays; asynchronous. */
int capgnn_cache_lookup(const capgnn_cache *c, const int64_t *ids, int64_t n, int by_gid,
                        int8_t *tier, int64_t *slot, void *stream);

typedef struct {
    int64_t hits;     /* rows served from the GPU tier  */
    int64_t misses;   /* rows served from the host tier */
    int64_t absent;   /* ids found in neither tier (rows zero-filled) */
} capgnn_gather_stats;

/* pick_cache: out[k, 0:dims[layer]] = table_layer[ids[k], :] as a bit copy.
 * ids: device int64[n] (halo-local indices, or global ids when by_gid), duplicates and any order
 * allowed; ids == NULL means "every halo vertex in halo-local order" (n must equal n_halo), the
 * case of full-batch training.  out: device [n x ld] of the cache's dtype.
 * GPU-tier rows are copied on `stream`.  Host-tier rows are moved on `side_stream` when it is
 * non-NULL (it first waits for everything enqueued on `stream` so far; `stream` then waits for the
 * transfer before the call returns control of `out` to later work on `stream`), else on `stream`.
 * staging: device scratch of capgnn_cache_sizes().staging_bytes for CAPGNN_MISS_STAGED, or NULL to
 * read pinned memory directly from the kernel (CAPGNN_MISS_ZEROCOPY).
 * stats != NULL forces a stream synchronisation and fills the counters.
 * Absent ids give zero rows and CAPGNN_ENOTFOUND (only detectable when stats != NULL). */
int capgnn_halo_gather(capgnn_cache *c, int layer, const int64_t *ids, int64_t n, int by_gid,
                       void *out, int64_t ld, void *stream, void *side_stream, void *staging,
                       capgnn_gather_stats *stats);

/* Vertex update (sections "Vertex Importance and Vertex Update" and "Staleness in CaPGNN": cached halo
 * representations are overwritten by newer ones and must not stay stale for an unbounded number of
 * iterations).  For k = 0..n-1: the cached row of ids[k] in `layer`'s table becomes rows[k, 0:dims[layer]], in
 * whichever tier holds it (GPU-tier rows are written in device memory, host-tier rows through the pinned
 * mapping), and is stamped with `epoch`.  Of several updates of one vertex in a call the last one stays.  No
 * lock is taken: rows and stamps of a call become visible together, in stream order, to the gathers and
 * epochs enqueued after it (the lock-free update of the section "Pipeline Design"; there is no reader inside
 * this library that runs concurrently with an update on the same stream).
 * ids: device int64[n] (halo-local indices, or global ids when by_gid); rows: device [n x ld] of the cache's
 * dtype.  Absent ids are skipped.  Asynchronous on `stream` unless stats != NULL (then it synchronises and
 * reports hits = rows written to the GPU tier, misses = rows written to the host tier, absent).
 * In CAPGNN_MISS_PIPELINED mode the copy of the host tier that the last capgnn_epoch prefetched stays valid: every
 * host-tier row written here is written into that copy too (the call first waits for a prefetch still in flight),
 * so the next epoch consumes the new rows without fetching the table again; `stream` must be ordered before that
 * epoch's stream.  That copy lives in the ws last passed to capgnn_epoch, which therefore must still be allocated: a
 * caller that frees or reuses that ws while updates may follow calls capgnn_cache_set_miss_mode first (it forgets the
 * copy).  Every table starts with stamp 0 (capgnn_cache_fill resets the layer's stamps to 0). */
int capgnn_cache_update(capgnn_cache *c, int layer, const int64_t *ids, int64_t n, int by_gid,
                        const void *rows, int64_t ld, int64_t epoch, void *stream,
                        capgnn_gather_stats *stats);

/* Bounded staleness: the halo-local indices h (ascending) of `layer`'s rows with epoch_now - stamp[h] > max_age,
 * i.e. the rows a periodic synchronisation has to refresh.  ids_out: device int64[n_halo]; *n_out (host) = how
 * many; *oldest (host, may be NULL) = the smallest stamp.  Synchronises `stream`. */
int capgnn_cache_stale(capgnn_cache *c, int layer, int64_t epoch_now, int64_t max_age,
                       int64_t *ids_out, int64_t *n_out, int64_t *oldest, void *stream);

/* Vertex overlap ratio, Eq. 2: R[v] = number of partitions whose halo set contains v.  halo_ids: device
 * int64[n_ids], the halo sets of all partitions one after another (every set duplicate-free; ids outside
 * [0, n_vertices) are ignored); R: device int32[n_vertices], overwritten (0 for vertices in no halo set).
 * Asynchronous on `stream`. */
int capgnn_overlap_ratio(const int64_t *halo_ids, int64_t n_ids, int64_t n_vertices, int32_t *R, void *stream);

/* RAPA's vertex influence score, Eq. 6, of every column vertex v of the partition graph (local vertices have
 * outgoing and incoming neighbours, halo vertices only outgoing ones):
 *   S[v] = ( inv_sqrt_dout[v] * sum_{rows i with an entry (i,v)} inv_sqrt_din[i]
 *          + [v local] inv_sqrt_din[v] * sum_{entries (v,j) of row v} inv_sqrt_dout[j] ) * count[v].
 * inv_sqrt_din: device float[n_loc], 1/sqrt of the in-degrees the caller wants (Eq. 6: of the original graph);
 * inv_sqrt_dout: device float[n_cols], 1/sqrt of the out-degrees (Eq. 6: in the subgraph); count: device
 * float[n_cols], how often the vertex appears across subgraphs, or NULL (= 1); S: device float[n_cols].
 * Edge values and the graph's own scales are not used.  Asynchronous on `stream`. */
int capgnn_influence_score(const capgnn_graph *g, const float *inv_sqrt_din, const float *inv_sqrt_dout,
                           const float *count, float *S, void *stream);

/* ------------------------------------------------------------------------------------------
 * RAPA's subgraph adjustment (section "Resource-Aware Partitioning Algorithm": cost model Eq. 3-5, Alg. 2
 * do_partition, Alg. 3 adjust_subgraph).  Host code; the ranking it consumes is capgnn_influence_score's (Eq. 6).
 * ---------------------------------------------------------------------------------------- */

/* One GPU as the cost model sees it: the measured cost (time) of the reference SpMM and MM and of the reference
 * transfer host-to-device, device-to-host and device-to-device (the paper measures them on a 11585 x 11585 matrix;
 * any unit, only the ratio to the largest value among the GPUs enters), and the memory available, in bytes. */
typedef struct {
    double t_spmm, t_mm;
    double f_h2d, f_d2h, f_idt;
    double mem_bytes;
} capgnn_rapa_device;

typedef struct {
    double alpha;        /* Eq. 4: weight of the SpMM term (edges) against the MM term (inner vertices), in [0,1] */
    double epsilon;      /* Alg. 2 stops when the standard deviation of the costs is below it                      */
    double m_vertex, m_edge, m_feat;  /* Eq. 5: bytes per vertex, per edge, per feature element                    */
    int64_t f_dim;       /* Eq. 5: feature width (the feature term counts f_dim elements for every vertex)          */
    double beta;         /* Eq. 5: bytes reserved for gradients and the like                                        */
    int max_sweeps;      /* safety bound on the sweeps of Alg. 2 (> 0)                                              */
} capgnn_rapa_params;

/* Edges of a partition graph by the kind of their source: *e_inner = entries whose column is a local vertex,
 * halo_edges[k] = entries whose column is halo vertex k (all of them outer edges).  Host arrays. */
int capgnn_halo_edge_counts(int64_t n_loc, int64_t n_halo, const int64_t *rowptr, const int32_t *col,
                            int64_t *e_inner, int64_t *halo_edges);

/* Alg. 2 around Alg. 3.  Subgraph i (on GPU i) has n_inner[i] inner vertices, e_inner[i] edges between them, and the
 * halo vertices halo_ptr[i] .. halo_ptr[i+1]-1 of the flat arrays halo_edges (edges of that halo vertex in the
 * subgraph) and score (its influence score S_k, Eq. 6, as computed by capgnn_influence_score).
 * lambda_i = alpha |E_all| t_spmm/tmax + (1-alpha) |V_inner| t_mm/tmax
 *          + |E_outer| ((f_h2d/fmax + f_d2h/fmax)(1 - 1/P) + f_idt/fmax / P)                     (Eq. 3, Eq. 4)
 * Every sweep (Alg. 3) visits the GPUs from the weakest on (largest alpha t_spmm/tmax + (1-alpha) t_mm/tmax, ties by
 * index).  A subgraph whose cost is at most the mean of all costs and whose memory suffices (Eq. 5) is marked done
 * (r_i = 1).  Otherwise its halo vertices are taken in ascending score order (ties by index; a vertex is considered
 * once over all sweeps) and removed with all their edges while the estimated cost exceeds the mean, stopping early once
 * it is at most halfway between the old cost and the mean and the memory suffices; if nothing was removed, r_i = 1.
 * The sweeps end (Alg. 2) when the standard deviation of the costs is below epsilon, when r = 1, or after max_sweeps.
 * Outputs (host): keep[halo_ptr[P]] = 1 for the halo vertices that stay; lambda_out[P]; r_out[P] (last sweep);
 * *sweeps_out; *sigma_out (after the last sweep); any of the last four may be NULL.
 * Costs are formed in double precision exactly as written above (no fused operations).  Errors: CAPGNN_EINVAL. */
int capgnn_rapa_adjust(int n_parts, const int64_t *n_inner, const int64_t *e_inner, const int64_t *halo_ptr,
                       const int64_t *halo_edges, const float *score, const capgnn_rapa_device *dev,
                       const capgnn_rapa_params *prm, uint8_t *keep, double *lambda_out, int32_t *r_out,
                       int *sweeps_out, double *sigma_out);

/* The subgraph without the halo vertices that keep[] drops ("Remove V_rem and E_rem from G_i", Alg. 3): their entries
 * disappear, the halo vertices that stay are renumbered in their old order.  rowptr_out: host int64[n_loc+1]; col_out:
 * host int32[nnz] (the first rowptr_out[n_loc] are written); new_index: host int64[n_halo], the new halo-local index
 * of each old halo vertex, -1 if dropped (the caller moves its halo attributes and cache rows alike). */
int capgnn_prune_halo(int64_t n_loc, int64_t n_halo, const int64_t *rowptr, const int32_t *col, const uint8_t *keep,
                      int64_t *rowptr_out, int32_t *col_out, int64_t *new_index);

#define CAPGNN_POLICY_JACA      0  /* static contents, highest overlap ratio first (ties: ascending vertex id) */
#define CAPGNN_POLICY_JACA_LOW  1  /* the same with the lowest overlap ratio first (the evaluation's counter-test) */
#define CAPGNN_POLICY_FIFO      2
#define CAPGNN_POLICY_LRU       3

/* Two-level cache policy comparison (evaluation sections "Impact of Vertex Overlap Ratio on Cache Hit Rate" and
 * "Impact of Cache Capacity and Partition on Cache Hit Rate": JACA against FIFO and LRU on one local cache per
 * partition plus one shared global cache).  Host only.  In every epoch the partitions take turns; partition i
 * requests every vertex of its halo set halo_ids[halo_ptr[i] .. halo_ptr[i+1]) (ascending, duplicate-free) in
 * that order.  A request is served by the partition's local cache, else by the global cache, else it is a miss.
 * JACA: local cache i holds the cap_local vertices of H_i with the highest overlap ratio, the global cache the
 * cap_global vertices of the union with the highest ratio.  FIFO / LRU: both levels start empty; a global hit or
 * a miss inserts the vertex into the local cache, a miss also into the global cache, evicting the
 * first-inserted / least-recently-used entry of a full cache.  Requests of the first `warmup` epochs are not
 * counted.  counts[3] (host) = local hits, global hits, misses. */
int capgnn_policy_simulate(int n_parts, const int64_t *halo_ptr, const int64_t *halo_ids, int policy,
                           int64_t cap_local, int64_t cap_global, int epochs, int warmup, int64_t *counts);

/* ------------------------------------------------------------------------------------------
 * Storage order of the vertices (the subgraph reordering that follows RAPA; the reorder figure).  The paper
 * names no algorithm, so any order is admissible as long as results only move with their vertex.  Host code.
 *
 * capgnn_locality_order: new2old[n_loc + n_halo] (host, written) = the vertex to store at each place; local
 * vertices keep places [0, n_loc), halo vertices the places after them.
 *   CAPGNN_RELABEL_POPULARITY  inside each range, vertices referenced by more entries first (ties: lower index)
 *   CAPGNN_RELABEL_BFS         local vertices in breadth-first order over the local-to-local entries: a search
 *                              starts at the unreached vertex with the longest row (ties: lower index) and scans
 *                              rows in stored order; halo vertices in the order in which the rows, walked in
 *                              the new local order, first mention them; unmentioned ones last, by index.
 * capgnn_relabel_csr: the CSR with vertices moved to those places: row k of the result is old row new2old[k]
 * with columns renumbered and its entries (edge_val with them, may be NULL) sorted by the new column, equal
 * columns in their old order: a sorted CSR stays sorted, a symmetric one equal to its transpose.  Outputs are host
 * arrays of the input's sizes, owned by the caller.  The caller moves the rows of its features, labels, masks
 * and halo attributes the same way (row k <- old row new2old[k]).
 * Errors: CAPGNN_EINVAL for malformed CSR, an unknown method, or a new2old that is no such permutation.
 * ---------------------------------------------------------------------------------------- */
#define CAPGNN_RELABEL_POPULARITY 0
#define CAPGNN_RELABEL_BFS 1
int capgnn_locality_order(int method, int64_t n_loc, int64_t n_halo, const int64_t *rowptr, const int32_t *col,
                          int32_t *new2old);
int capgnn_relabel_csr(int64_t n_loc, int64_t n_halo, const int64_t *rowptr, const int32_t *col,
                       const float *edge_val, const int32_t *new2old, int64_t *rowptr_out, int32_t *col_out,
                       float *val_out);

/* ------------------------------------------------------------------------------------------
 * Dense products on the matrix cores (the combination step; the MM term of RAPA's cost model, Eq. 4).
 * C[M x N] (+)= op(A) op(B) with fp32 accumulation; optional fused bias / ReLU epilogue.
 * trans_a: A is stored [K x M];  trans_b: B is stored [N x K].  bias: device float[N] or NULL.
 * relu_mask: device [M x ldm] of `dtype` or NULL; when given, C[i,j] is zeroed where
 * relu_mask[i,j] <= 0 (the sigma' factor of the backward recursion).
 * ws is required when trans_a (reduction over the vertex dimension is split over workgroups and
 * reduced in a fixed order) and optional otherwise (room to lay the weight matrix out for the bf16
 * matrix cores; without it a slower kernel runs): capgnn_gemm_workspace_bytes().
 * out_f32 != 0 stores C as float even when dtype is BF16 (weight gradients, logits).
 * The padding of operand rows (columns beyond the operand's width, inside its ld) may be read, whatever it holds, but
 * never reaches C; nothing is read beyond the last row's width.  Padding columns of C are not written.
 * ---------------------------------------------------------------------------------------- */
size_t capgnn_gemm_workspace_bytes(int trans_a, int64_t M, int64_t N, int64_t K);

/* How a product of fp32 operands is formed: an argument of capgnn_gemm and a field of capgnn_layer (nothing is
 * process-wide, so distinct handles and calls stay independent).
 *   CAPGNN_F32_PRODUCT_AUTO    (0, what a zeroed field means) SPLIT for products of 2^28 multiply-adds and more, except
 *                              trans_a products with N <= 64; NATIVE otherwise.
 *   CAPGNN_F32_PRODUCT_NATIVE  the fp32 matrix instruction (v_mfma_f32_32x32x2_f32).
 *   CAPGNN_F32_PRODUCT_SPLIT   each fp32 operand is cut, exactly, into three bf16 numbers and the six largest of the nine
 *                              piece products are accumulated in fp32 on the bf16 matrix cores; what is dropped is
 *                              2^-23 of a product at most, the size of the fp32 instruction's own rounding.  Needs the
 *                              workspace of capgnn_gemm_workspace_bytes() also when !trans_a (the weight matrix is cut
 *                              there); without it, and for trans_a && trans_b, the native instruction runs.
 *                              Non-finite operands give NaN where the native instruction may give an infinity.
 * bf16 operands are not affected.  Any other value: CAPGNN_EINVAL. */
#define CAPGNN_F32_PRODUCT_AUTO 0
#define CAPGNN_F32_PRODUCT_NATIVE 1
#define CAPGNN_F32_PRODUCT_SPLIT 2

/* Measurement aid for the matrix-core roofline of the dense products: launches `workgroups` workgroups of 256 threads
 * that each issue 4 * iters register-resident matrix instructions per wave (v_mfma_f32_32x32x2_f32 for CAPGNN_F32,
 * v_mfma_f32_32x32x16_bf16 for CAPGNN_BF16) and returns in *flop (host) the floating-point operations the launch
 * performs; the caller times it.  out: device float[workgroups * 256] (receives one value per thread). */
int capgnn_mfma_peak(int dtype, int workgroups, int iters, float *out, double *flop, void *stream);

/* Measurement aid for the gather roofline of the aggregation: `workgroups` workgroups of 256 threads whose 8-lane groups
 * each fetch 16 * iters pseudo-random 128-byte lines (16 bytes per lane, 16 loads in flight) out of table_lines
 * lines that lie line_stride lines apart in `table` (device, table_lines * line_stride * 128 bytes, 16-byte aligned;
 * table_lines a power of two, at most 2^24; line_stride 1 = a dense table, 9 = the slices of rows with a pitch of nine
 * lines), and nothing else.  *bytes (host) = the bytes the launch requests; the
 * caller times it.  With a table that fits an L2 (4 MB per XCD), the Infinity Cache (256 MB) or neither, the rate is
 * what that level delivers for the aggregation's access pattern.  out: device float[workgroups * 256]. */
int capgnn_gather_peak(const void *table, int64_t table_lines, int line_stride, int workgroups, int iters, float *out,
                       double *bytes, void *stream);
int capgnn_gemm(int trans_a, int trans_b, int64_t M, int64_t N, int64_t K,
                const void *A, int64_t lda, const void *B, int64_t ldb, void *C, int64_t ldc,
                int dtype, int out_f32, int accumulate, const float *bias, int relu,
                const void *relu_mask, int64_t ldm, int f32_product, void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------------------------
 * Layer and epoch.
 * ---------------------------------------------------------------------------------------- */
typedef struct {
    int kind;            /* CAPGNN_GCN | CAPGNN_SAGE_MEAN                                   */
    int f_in, f_out;
    int act;             /* CAPGNN_ACT_NONE | CAPGNN_ACT_RELU                               */
    int dtype;           /* storage type of X, H and of W / W_self                          */
    int order;           /* CAPGNN_ORDER_AUTO | CAPGNN_AGG_FIRST | CAPGNN_XFORM_FIRST       */
    int out_f32;         /* store H as float even when dtype is BF16 (the layer that feeds the loss) */
    int f32_product;     /* CAPGNN_F32_PRODUCT_*: how this layer's products of fp32 operands are formed (0 = AUTO) */
    void *W;             /* device [f_in x f_out], dense (ld = f_out); neighbour weight for SAGE */
    void *W_self;        /* device [f_in x f_out], SAGE only, else NULL                     */
    float *bias;         /* device float[f_out] or NULL                                     */
} capgnn_layer;

/* The association the library would use for this layer (resolves ORDER_AUTO with a byte/FLOP
 * cost model that includes the backward pass). */
int capgnn_layer_order(const capgnn_graph *g, const capgnn_layer *l, int need_dx);

/* Forward: H = act(A_hat X W + bias)            (GCN, proof of Lemma 2)
 *          H = act(X_loc W_self + mean_agg(X) W + bias)   (GraphSAGE-mean)
 * X: device [n_cols x ldx] = [local rows; halo rows]; H: device [n_loc x ldh].
 * saved: device buffer of capgnn_layer_saved_bytes() that layer_bwd needs (the aggregated input
 * for AGG_FIRST; nothing for XFORM_FIRST). */
size_t capgnn_layer_saved_bytes(const capgnn_graph *g, const capgnn_layer *l);
size_t capgnn_layer_workspace_bytes(const capgnn_graph *g, const capgnn_layer *l);
int capgnn_layer_fwd(const capgnn_graph *g, const capgnn_layer *l, const void *X, int64_t ldx,
                     void *H, int64_t ldh, void *saved, void *ws, size_t ws_bytes, void *stream);

/* Backward of the same layer.  H is the forward output (its sign pattern is sigma').  dH: device
 * [n_loc x lddh], gradient w.r.t. H, of the type H is stored in (float for a BF16 layer with out_f32: the loss
 * gradient is consumed unrounded - it is summed over all vertices, and values that cluster as closely as
 * (softmax - onehot) / n would all be rounded the same way); it is overwritten with dZ = dH * 1[H > 0] for ReLU layers, and its
 * contents afterwards are unspecified (a GCN layer of an operator without edge values leaves dZ with each row
 * multiplied by the row's normalisation scale, the form its transposed aggregation reads).
 * dW, dW_self: device float [f_in x f_out] (dense); dbias: device float[f_out]; any may be NULL.
 * dX: device [n_rows_dx x lddx] or NULL; n_rows_dx = n_cols when need_halo_grad, else n_loc
 * (gradient w.r.t. the halo rows is computed only on request; it is never sent anywhere). */
int capgnn_layer_bwd(const capgnn_graph *g, const capgnn_layer *l, const void *X, int64_t ldx,
                     const void *H, int64_t ldh, const void *saved, void *dH, int64_t lddh,
                     float *dW, float *dW_self, float *dbias, void *dX, int64_t lddx,
                     int need_halo_grad, void *ws, size_t ws_bytes, void *stream);

/* Masked softmax cross-entropy (evaluation setup: cross-entropy for single-label tasks) and its
 * gradient: loss = (1/norm) sum_{mask} (logsumexp(Z_i) - Z_i[y_i]); dZ_i = (softmax(Z_i)-e_y)/norm.
 * Z: device float [n x ldz] (C classes); labels: device int32[n]; mask: device uint8[n] or NULL;
 * loss_norm <= 0 means "number of masked rows".  loss_dev: device float[1].  dZ: device [n x lddz] of dz_dtype
 * (float, or bf16 so that a bf16 backward pass can consume it directly), or NULL.
 * Labels outside [0,C) are clamped into range.  ws: capgnn_loss_workspace_bytes(n). */
size_t capgnn_loss_workspace_bytes(int64_t n);
int capgnn_softmax_ce(int64_t n, int C, const float *Z, int64_t ldz, const int32_t *labels,
                      const uint8_t *mask, double loss_norm, float *loss_dev, void *dZ, int64_t lddz,
                      int dz_dtype, void *ws, size_t ws_bytes, void *stream);

/* For callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): capgnn_softmax_ce without the workspace arguments.  Its scratch is a device array built into the
 * library, sized for n <= CAPGNN_LOSS_STATIC_MAX_ROWS (4 MiB + 8 KiB per GPU, held until the process ends); more rows
 * return CAPGNN_ENOMEM and touch nothing.  The call allocates nothing and frees nothing, on the host or the device.
 * It runs on the CURRENT device, which must be the device of `stream`, Z, labels, mask, loss_dev and dZ.  All calls on
 * one GPU share that GPU's array: calls that may overlap in time on one GPU (different streams, or different
 * threads) race on it; calls on one stream are ordered and safe.  Results are those of capgnn_softmax_ce bit for bit. */
#define CAPGNN_LOSS_STATIC_MAX_ROWS (1 << 20)
int capgnn_softmax_ce_static(int64_t n, int C, const float *Z, int64_t ldz, const int32_t *labels,
                             const uint8_t *mask, double loss_norm, float *loss_dev, void *dZ, int64_t lddz,
                             int dz_dtype, void *stream);

/* Masked binary cross-entropy on logits (evaluation setup: binary cross-entropy for multi-label tasks) and its
 * gradient: loss = (1/norm) sum_{mask} sum_k ( max(z,0) - z*y + log(1 + exp(-|z|)) ), which equals
 * -[y log s(z) + (1-y) log(1 - s(z))] with s the logistic function; dZ = (s(Z) - Y)/norm, zero in unmasked rows.
 * targets: device uint8 [n x ldt], nonzero = the label is set.  loss_norm <= 0 means "masked rows x C" (the mean over
 * elements).  Other arguments, workspace and errors as capgnn_softmax_ce. */
int capgnn_sigmoid_bce(int64_t n, int C, const float *Z, int64_t ldz, const uint8_t *targets, int64_t ldt,
                       const uint8_t *mask, double loss_norm, float *loss_dev, void *dZ, int64_t lddz,
                       int dz_dtype, void *ws, size_t ws_bytes, void *stream);

#define CAPGNN_MAX_RECORDS 96
#define CAPGNN_K_GATHER_HIT   1
#define CAPGNN_K_GATHER_MISS  2
#define CAPGNN_K_SPMM_FWD     3
#define CAPGNN_K_SPMM_BWD     4
#define CAPGNN_K_GEMM         5
#define CAPGNN_K_LOSS         6
#define CAPGNN_K_ELEMENTWISE  7
#define CAPGNN_K_GATHER_STAGED 8   /* device copy of host-tier rows out of the staging area into the layer input */

typedef struct {
    /* stage names follow the evaluation's breakdown: check_cache, pick_cache, communication,
     * aggregation; `communication` here is the host-tier transfer on the side stream. */
    float total_ms, check_cache_ms, pick_cache_ms, communication_ms, aggregation_ms,
          combine_ms, loss_ms, other_ms;
    int n_records;
    struct { int kind, layer, backward; float ms; } records[CAPGNN_MAX_RECORDS];
} capgnn_epoch_times;

/* One full-batch epoch over the partition: for l = 0..L-1 { halo rows of layer l's input <- cache;
 * layer forward }, loss, for l = L-1..0 { layer backward }, optional W <- W - lr*dW (update rule in
 * the proof of the convergence theorem).
 *   X0: device [n_cols x ld0]; rows [0,n_loc) hold the local input features, rows [n_loc,n_cols)
 *       are filled by this call from the cache's layer-0 table.
 *   c: NULL iff n_halo == 0.  labels/mask: device.  logits: device float [n_loc x f_out(L-1)] dense, or NULL.
 *   dW[l], dW_self[l], dbias[l]: device float buffers per layer (dW_self[l] NULL for GCN).
 *   loss_out: host float*, written after a stream synchronisation (the only forced sync);
 *   times: NULL, or filled from HIP events recorded on the streams the kernels run on (adds a sync).
 *   ws: capgnn_epoch_workspace_bytes(); side_stream may be NULL (then everything runs on `stream`).
 * Errors: EINVAL, ENOMEM (workspace too small), EUNSUPPORTED, EHIP. */
size_t capgnn_epoch_workspace_bytes(const capgnn_graph *g, const capgnn_cache *c,
                                    const capgnn_layer *layers, int L);
int capgnn_epoch(const capgnn_graph *g, capgnn_cache *c, const capgnn_layer *layers, int L,
                 void *X0, int64_t ld0, const int32_t *labels, const uint8_t *mask, double loss_norm,
                 float *logits, float **dW, float **dW_self, float **dbias, float lr,
                 float *loss_out, capgnn_epoch_times *times,
                 void *ws, size_t ws_bytes, void *stream, void *side_stream);

/* The same epoch for a multi-label task: the loss is capgnn_sigmoid_bce on targets (device uint8 [n_loc x ldt])
 * instead of the softmax cross-entropy on labels.  Everything else as capgnn_epoch. */
int capgnn_epoch_multilabel(const capgnn_graph *g, capgnn_cache *c, const capgnn_layer *layers, int L,
                            void *X0, int64_t ld0, const uint8_t *targets, int64_t ldt, const uint8_t *mask,
                            double loss_norm, float *logits, float **dW, float **dW_self, float **dbias, float lr,
                            float *loss_out, capgnn_epoch_times *times,
                            void *ws, size_t ws_bytes, void *stream, void *side_stream);

/* Where capgnn_epoch leaves the output of hidden layer l (0 <= l < L-1) inside ws: *ptr = device
 * address of H_l ([n_loc x *ld] of the layers' dtype), valid until ws is reused.  Same arguments as
 * capgnn_epoch_workspace_bytes; no GPU work.  For callers that want the embeddings, and for tests. */
int capgnn_epoch_activation(const capgnn_graph *g, const capgnn_cache *c, const capgnn_layer *layers, int L,
                            int l, void *ws, void **ptr, int64_t *ld);

/* The same epoch recorded once as a HIP graph and replayed with one launch per epoch: for partitions whose epoch is a
 * few dozen short kernels and therefore bound by their launches (the smallest evaluation graphs), and to take the
 * launch gaps out of any epoch.  Arguments as capgnn_epoch, except: `stream` is required and not the default stream;
 * no host loss and no event times; loss_dev: device float that every replay writes the loss to, or NULL.
 * side_stream NULL: everything is recorded on `stream`, host-tier rows travel inside the epoch that consumes them,
 * whatever the miss mode.  side_stream given: the two-stream epoch is recorded as it runs; in CAPGNN_MISS_PIPELINED
 * mode every replay consumes the host-tier rows that the run before it prefetched and prefetches for the next one, so
 * one capgnn_epoch with the same ws and side stream must have run before the recording (EINVAL otherwise), and a
 * replay ends only when its prefetches have.
 * The graph holds the ADDRESSES of every buffer given here (X0, labels, mask, logits, dW / dW_self / dbias and the
 * arrays of pointers' targets, the layers' weights, ws, the cache's tiers): they must stay allocated and in place
 * until the graph is destroyed; their CONTENTS may change between replays (new features, capgnn_cache_update /
 * capgnn_cache_fill - after which one eager capgnn_epoch primes the prefetch again -, the SGD step of the epoch itself
 * when lr != 0).  create: records without running (the buffers are not touched); launch: asynchronous on `stream` (any
 * stream of the same device; replays must not overlap one another or an eager epoch on the same ws); destroy: after the
 * last replay has finished.  The graph contains kernels and copies only.  Errors: as capgnn_epoch, EHIP if capture or
 * instantiation fail. */
typedef struct capgnn_epoch_graph capgnn_epoch_graph;
int capgnn_epoch_graph_create(capgnn_epoch_graph **out, const capgnn_graph *g, capgnn_cache *c,
                              const capgnn_layer *layers, int L, void *X0, int64_t ld0, const int32_t *labels,
                              const uint8_t *mask, double loss_norm, float *logits, float **dW, float **dW_self,
                              float **dbias, float lr, float *loss_dev, void *ws, size_t ws_bytes, void *stream,
                              void *side_stream);
int capgnn_epoch_graph_launch(capgnn_epoch_graph *eg, void *stream);
int capgnn_epoch_graph_destroy(capgnn_epoch_graph *eg);

#ifdef __cplusplus
}
#endif
#endif /* CAPGNN_H */
