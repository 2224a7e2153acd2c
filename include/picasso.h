/* picasso.h -- C-ABI of the MI355X (gfx950) mesh-decimation library.
 *
 * Implements the round-based QEM decimation of the Picasso paper
 * (Sec. 3, Algorithm 2 "Fast GPU-accelerated mesh simplification";
 * supplementary section "Quadric error computation"), and around it the
 * operators the paper defines on its results: pooling and unpooling over the
 * vertex clusters (Sec. 3), the replace / mapping tensors, and the
 * vertex2facet / facet2facet / facet2vertex convolutions (Sec. 4).  Every step runs in
 * hand-written HIP kernels; there is no CPU fallback.
 *
 * Conventions for every call
 *   - d_*   : DEVICE pointers owned by the caller; h_* / plain scalars: HOST.
 *   - verts : float32 [N,3] row-major.  facets: int32 [F,3] row-major.
 *   - return 0 = OK, >0 = warning, <0 = error (see picasso_status).
 *     On error no output buffer has been written.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  The
 *     decimate calls return when everything they queued on that stream has been
 *     done: all outputs are complete (they wait for their last kernel, see
 *     PICASSO_OPT_HOST_POLL).
 *   - A context owns its scratch workspace, a small pinned host buffer that its
 *     kernels write counters into, and one internal stream of default priority;
 *     it is bound to one device, which the calls make current; calls on one
 *     context must not overlap in time.  Contexts share no state: different
 *     contexts may be used from different host threads at the same time.
 *     Inputs are never modified.
 *   - Nothing is allocated inside the decimate calls.
 */
#ifndef PICASSO_H
#define PICASSO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct picasso_ctx picasso_ctx;

enum picasso_status {
    PICASSO_OK = 0,
    PICASSO_WARN_BUDGET_UNMET = 1, /* some mesh ran out of edges: its nv_out > target_nv          */
    PICASSO_ERR_INVALID_ARG = -1,  /* null pointer, N < 1, F < 0, target_nv < 1, B < 1              */
    PICASSO_ERR_BAD_INDEX = -2,    /* facet index outside [0,N) (batched: outside its own mesh)     */
    PICASSO_ERR_NONFINITE = -3,    /* NaN or Inf vertex coordinate                                  */
    PICASSO_ERR_WORKSPACE = -4,    /* input larger than the context was created for                 */
    PICASSO_ERR_HIP = -5,          /* HIP runtime error (see picasso_last_hip_error)                */
    PICASSO_ERR_INTERNAL = -6      /* a kernel met sizes that its launch does not take: a defect of
                                      the library, never of the input; outputs unspecified          */
};

enum picasso_option {
    PICASSO_OPT_MAX_ROUNDS = 0,    /* stop after this many runs of the core algorithm; <0 = no cap  */
    PICASSO_OPT_STAGE_TIMING = 1,  /* 1: fill picasso_stats.ms_stage with hipEvent times (slower)    */
    PICASSO_OPT_SUBROUND_BATCH = 2,/* selection sub-rounds launched between two host checks         */
    PICASSO_OPT_KERNEL_TIMING = 3, /* N > 0: in every N-th decimate call from now on, bracket the
                                      launches of the path's largest kernels with hipEvents
                                      (see picasso_kernel_timing); an event pair costs several
                                      microseconds of queue time per launch, and such a call keeps
                                      all its work on `stream` (as with PICASSO_OPT_OVERLAP 0), so
                                      that a bracketed kernel runs alone on the chip; 0: off       */
    PICASSO_OPT_OVERLAP = 4,       /* 1 (default): for inputs of 2^18 facets or more, the first
                                      round's edge-key sort runs on a stream of the context's own
                                      beside the vertex quadrics and joins `stream` before costs
                                      are computed; 0: everything on `stream`                      */
    PICASSO_OPT_TRUNC_BLOCK_MAX = 5,/* budget step (Alg. 2 lines 3-4 and 6): a mesh that formed more
                                      pairs than it may remove keeps its cheapest ones; while no
                                      such mesh formed more than this many pairs (default and
                                      largest value 32768) one workgroup per mesh selects them,
                                      above it the pairs of all such meshes are sorted.  Same
                                      result either way.                                           */
    PICASSO_OPT_PLACEMENT = 6,     /* where a pair is contracted to, and where its cost is taken
                                      (Alg. 2 lines 2 and 14; supplementary, the two placement
                                      equations).  0 (default): the mean of the two positions.
                                      1: the point of least quadric error, the solution of
                                      A x = -b for the pair's summed quadric, wherever A is of
                                      full rank, else the mean.  A (positive semi-definite) is
                                      factored with diagonal pivoting; it counts as of full rank
                                      when its three pivots are positive and smallest / largest
                                      exceeds the threshold below (the paper tests the reciprocal
                                      condition number without saying how or against what).      */
    PICASSO_OPT_RCOND_MIN_BITS = 7,/* that threshold, passed as the bit pattern of a binary32
                                      value (finite, >= 0; default 1e-3)                          */
    PICASSO_OPT_ABSORB = 8,        /* 1: Alg. 2 line 11 (Fig. 2 (c)) is applied in every run of the
                                      core algorithm, under the vertex budget: once the pairs
                                      are formed, a vertex in no pair that has an edge to a
                                      paired vertex joins that pair's cluster through its
                                      cheapest such edge (cost, edge index), cheapest vertices
                                      first, while the mesh may still lose vertices; a vertex
                                      that joined attracts no others.  A cluster's quadric and
                                      mean position are summed over its members in ascending
                                      index order; it is represented by its pair's smaller
                                      index.  0 (default): pairs only.                           */
    PICASSO_OPT_SHUFFLE_SEED = 9,  /* the shuffle inserted into the sorting of the pairs (Sec. 3,
                                      footnote; Sec. 5, augmentation): with a seed != 0, pairs of
                                      equal cost are taken in the order of a seeded bijection of
                                      their 32-bit index (xor with the seed's low word, times
                                      0x9E3779B1, x ^= x >> 15, times 0x85EBCA77, x ^= x >> 13,
                                      plus the seed's high word) instead of index order; pairs
                                      of different cost keep their order.  All 64 bits of the
                                      value are the seed; 0 (default): index order.              */
    PICASSO_OPT_HOST_POLL = 10,    /* where a decimate call has to wait for the device (once per
                                      round, and at its end) the host watches a sequence number
                                      that a kernel stores in the context's pinned host memory
                                      after its results, for at most this many microseconds, and
                                      synchronises the stream if it has not come by then.  1
                                      (default) = 20,000 us; 0 = synchronise the stream at once;
                                      at most 10,000,000.  The results are the same either way.  */
    PICASSO_OPT_LAUNCH_AHEAD = 11, /* 1 (default): in a round of at most 2^20 facets in
                                      which the outcome of the selection decides nothing but
                                      counts (no mesh can exceed its budget, or some mesh surely
                                      will and the per-mesh budget step can take it), the kernels
                                      that follow the selection are queued behind it before the
                                      host has looked; they do nothing if the selection turns out
                                      to need more passes.  0: queued after the look.  Same
                                      results.                                                   */
    PICASSO_OPT_TRUNC_WIDTH = 12,  /* test hook for the per-mesh budget step: 0 (default) = its
                                      workgroups hold 4, 8, 16 or 32 cost keys per lane (x 1024
                                      lanes) as the largest mesh needs; 4, 8, 16 or 32 = always
                                      that many, so that a mesh with more pairs than fit makes
                                      the kernel report it and the call return
                                      PICASSO_ERR_INTERNAL instead of a wrong budget.            */
    PICASSO_OPT_DROP_DEGENERATED = 13, /* 1: degenerated vertices are removed (Sec. 3, "Pooling and
                                      unpooling": the mapping tensor's degenerated-vertex
                                      information; the paper leaves its definition to code it does
                                      not print).  An output vertex that no output facet refers
                                      to (its cluster no longer touches the surface; also an input
                                      vertex that never did) is dropped at the end of the call:
                                      the other output vertices keep their order and are
                                      renumbered, nv_out counts them (it may fall below target_nv),
                                      and d_cluster_id holds -1 for the input vertices of dropped
                                      clusters.  0 (default): every cluster stays an output vertex. */
    PICASSO_OPT_TRUNC_SELECT = 14  /* budget step (Alg. 2 lines 3-4 and 6) of a single mesh that
                                      formed more pairs than PICASSO_OPT_TRUNC_BLOCK_MAX, ties in
                                      index order: 1 (default) = the cost key at the budget is
                                      found by three histogram passes over the pairs' cost keys;
                                      0 = the pairs are sorted, as they are for a batch or with a
                                      shuffle seed.  Same results.                               */
};

#define PICASSO_STATS_ROUNDS 32
enum picasso_stage { /* index into picasso_stats.ms_stage[round][...] */
    PICASSO_ST_QUADRICS = 0, /* S0, round 0 only */
    PICASSO_ST_EDGES = 1,    /* S1 emit + sort + unique (+ fused S2 cost) */
    PICASSO_ST_SELECT = 2,   /* S3 sub-rounds (+ budget truncation, S2b) */
    PICASSO_ST_CONTRACT = 3, /* S4 + S6 vertex side */
    PICASSO_ST_FACETS = 4,   /* S5 facet clean-up + compaction */
    PICASSO_ST_COUNT = 8
};

typedef struct picasso_stats {
    int32_t rounds;                          /* runs of the core algorithm executed                 */
    int32_t nv_out, nf_out;                  /* totals over all meshes                              */
    int32_t nv[PICASSO_STATS_ROUNDS];        /* vertices entering round r                           */
    int32_t nf[PICASSO_STATS_ROUNDS];        /* facets entering round r                             */
    int32_t ne[PICASSO_STATS_ROUNDS];        /* distinct edges in round r                           */
    int32_t nsel[PICASSO_STATS_ROUNDS];      /* vertices removed in round r (pairs; + joiners of line 11) */
    int32_t subrounds[PICASSO_STATS_ROUNDS]; /* selection sub-rounds launched in round r            */
    float ms_stage[PICASSO_STATS_ROUNDS][PICASSO_ST_COUNT];
    float ms_total;                          /* whole call, hipEvents on `stream`                   */
} picasso_stats;

/* Bytes of device workspace a context of this capacity allocates. */
size_t picasso_workspace_bytes(int64_t max_verts, int64_t max_facets, int32_t max_meshes);

/* Create a context on `device` able to decimate up to max_verts vertices,
 * max_facets facets (totals over a batch) and max_meshes meshes per call.
 * Limits (32-bit indices): max_verts < 2^31 - 16, max_facets <= 2^29, else
 * PICASSO_ERR_INVALID_ARG.  Allocates the workspace and a small pinned host
 * buffer once; returns PICASSO_ERR_HIP if that fails. */
int picasso_create(picasso_ctx** out, int device, int64_t max_verts, int64_t max_facets, int32_t max_meshes);
void picasso_destroy(picasso_ctx* ctx);
int picasso_set_option(picasso_ctx* ctx, int option, int64_t value);
const char* picasso_strerror(int status);
const char* picasso_last_hip_error(picasso_ctx* ctx);

/* Kernels whose launches PICASSO_OPT_KERNEL_TIMING brackets with hipEvents, and the algorithmic
 * bytes a launch of each is charged with (what the step has to move at least, from the sizes of the
 * round it runs in: nv vertices, nf facets, H = 3 nf half-edges, E distinct edges; N, F = the call's
 * input sizes):
 *   SORT          per-bucket kernel of the 64-bit edge-key sort (Alg. 2 line 1; the scatter passes
 *                 when an input beyond 2^23 keys falls back to plain radix passes): every 8-byte
 *                 key read and written once, 16 H.
 *   UNIQUE_COST   distinct edges, their costs (Alg. 2 line 2) and first bids: 8 H (sorted keys
 *                 read) + 13 E (edge key, cost key, state written) + 64 nv (every vertex record
 *                 read once) + 8 nv (one bid word per vertex).
 *   SUBROUND0     first grid-wide sub-round of the selection (Alg. 2 lines 3-10): 13 E read, E
 *                 written (edge states), 3 x 8 nv (bids read, next bids written, third array cleared).
 *   FACET_INSERT  facets re-indexed and entered into the hash set, cluster labels composed:
 *                 12 nf read + 12 nf re-indexed + 4 nf deciding slot + 4 nf table slot + 4 nv
 *                 (vertex map) + 8 N (labels read and written).
 *   QUADRIC_ROWS  vertex quadrics summed from the facets' planes (supplementary, vertex quadric
 *                 equation): 8 x 3F sorted incidences + 16 F planes + 12 N positions + 64 N records.
 *   SORT_INCIDENCE per-bucket kernel of the sort that brings the 3F (vertex, facet) incidence keys
 *                 into vertex order for the vertex quadrics (once per call): 16 x 3F. */
enum picasso_timed_kernel {
    PICASSO_KERNEL_SORT = 0,
    PICASSO_KERNEL_UNIQUE_COST = 1,
    PICASSO_KERNEL_SUBROUND0 = 2,
    PICASSO_KERNEL_FACET_INSERT = 3,
    PICASSO_KERNEL_QUADRIC_ROWS = 4,
    PICASSO_KERNEL_SORT_INCIDENCE = 5,
    PICASSO_KERNEL_COUNT = 6
};

/* Totals gathered for `kernel` while PICASSO_OPT_KERNEL_TIMING is on, over all decimate calls
 * since the last reset: launches, their summed hipEvent time, their summed algorithmic bytes.
 * Host pointers, may be NULL.  reset != 0 clears that kernel's totals afterwards. */
int picasso_kernel_timing(picasso_ctx* ctx, int kernel, int reset, int64_t* launches, double* ms_total,
                          double* bytes_total);

/* Alg. 2 repeated until the vertex budget is met (Sec. 3: "running the core
 * algorithm multiple times").
 *
 *   d_verts [N,3], d_facets [F,3]          inputs
 *   target_nv                              number of output vertices N of Alg. 2
 *   d_verts_out  (capacity N*3 floats)     contracted positions, first nv_out rows
 *   d_facets_out (capacity F*3 ints)       surviving facets re-indexed, first nf_out rows,
 *                                          input order and winding kept
 *   d_cluster_id [N]                       output vertex that replaces each input vertex
 *                                          (the paper's 1-D vertex-clustering tensor)
 *   h_nv_out, h_nf_out                     host scalars
 *   stats                                  host, may be NULL
 *
 * One round = Alg. 2 lines 1-10 and 12-16 with pairs only: distinct mesh edges
 * are the candidates (line 1); pair cost = summed vertex quadrics evaluated at
 * the pair's mean (line 2, supplementary Q(x) and mean-placement equations);
 * pairs are taken greedily in ascending (cost, edge index) order while both
 * ends are free and fewer than |V|-target pairs were taken (lines 3-10); each
 * pair is contracted to its mean with the summed quadric, the smaller index
 * representing it (lines 12-16).  Facets with two equal indices and later
 * copies of an identical vertex triple are removed; survivors are renumbered
 * in ascending order.  target_nv >= N copies the input through unchanged.
 */
int picasso_decimate(picasso_ctx* ctx, void* stream, const float* d_verts, int32_t N, const int32_t* d_facets,
                     int32_t F, int32_t target_nv, float* d_verts_out, int32_t* d_facets_out,
                     int32_t* d_cluster_id, int32_t* h_nv_out, int32_t* h_nf_out, picasso_stats* stats);

/* Same on B concatenated meshes (Sec. 3: "mini-batches of concatenated
 * meshes"): mesh b owns vertices [sum nv_in[<b], +nv_in[b]) and the facets
 * [sum nf_in[<b], +nf_in[b]), whose indices are GLOBAL and must stay inside the
 * mesh's own vertex range.  Budgets are per mesh.  Outputs are concatenated in
 * mesh order with global output indices; h_nv_out/h_nf_out are host arrays [B].
 * The result equals decimating every mesh on its own. */
int picasso_decimate_batch(picasso_ctx* ctx, void* stream, int32_t B, const float* d_verts, const int32_t* d_facets,
                           const int32_t* h_nv_in, const int32_t* h_nf_in, const int32_t* h_target_nv,
                           float* d_verts_out, int32_t* d_facets_out, int32_t* d_cluster_id, int32_t* h_nv_out,
                           int32_t* h_nf_out, picasso_stats* stats);

/* ---- pooling / unpooling over the clusters (Sec. 3, "Pooling and unpooling") ----
 *
 * The clusters recorded in cluster_id are the pooling neighbourhoods.  Features
 * are float32 [N, C] row-major device arrays.  Sums run over a cluster's members
 * in ascending vertex order, left to right in fp32, without fp atomics, so the
 * results are reproducible to the bit. */

enum picasso_pool_mode {
    PICASSO_POOL_AVG = 0,      /* y_c = (sum_v x_v) / |c|                                          */
    PICASSO_POOL_MAX = 1,      /* y_c = max_v x_v per channel; argmax = first member attaining it   */
    PICASSO_POOL_WEIGHTED = 2, /* y_c = (sum_v w_v x_v) / (sum_v w_v), 0 if the weights sum to 0    */
    PICASSO_POOL_SUM = 3       /* y_c = sum_v x_v                                                   */
};

/* The two 1-D tensors of input-vertex length in Alg. 2's output list (Sec. 3,
 * "Pooling and unpooling": clustering and degenerated-vertex information; the
 * paper leaves their definition to code it does not print), derived from a
 * decimate call's d_cluster_id: d_replace[v] = representative of v's cluster as
 * an input vertex index (the cluster's smallest member), d_mapping[v] = output
 * index of v if v is that representative, else -1, so that
 * d_cluster_id[v] == d_mapping[d_replace[v]]; a vertex with cluster id -1 (its cluster was dropped, see
 * PICASSO_OPT_DROP_DEGENERATED) gets -1 in both.  Device pointers of n_in ints
 * each, owned by the caller.  Waits for its work on the stream (as the decimate
 * calls do); returns
 * PICASSO_ERR_BAD_INDEX (outputs then unspecified) if an id lies outside
 * [-1, n_out).  0 <= n_out <= max_verts of the context. */
int picasso_replace_mapping(picasso_ctx* ctx, void* stream, const int32_t* d_cluster_id, int32_t n_in, int32_t n_out,
                            int32_t* d_replace, int32_t* d_mapping);

/* For callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): picasso_replace_mapping
 * without a context.  The one scratch array the two kernels need (the smallest
 * member of every cluster, n_out ints, and an error flag) lives in a static
 * device array inside the library, so n_out <= PICASSO_STATIC_MAX_CLUSTERS
 * (16 MiB per device, held until the process ends); a larger n_out returns
 * PICASSO_ERR_WORKSPACE and nothing is queued.  The call allocates nothing
 * (no hipMalloc / hipFree, no allocating library routine), creates no stream or
 * event, does not wait and uses no pinned host memory: it queues three kernels
 * on `stream` of `device` (0 <= device < 64) and returns.  Instead of a status
 * that would need a wait, the last kernel stores PICASSO_OK or
 * PICASSO_ERR_BAD_INDEX (an id outside [0, n_out); d_replace / d_mapping then
 * unspecified) in the device word d_status; the return value covers the
 * argument checks and launch errors only.  d_replace, d_mapping [n_in],
 * d_status [1]: device memory owned by the caller; same results as
 * picasso_replace_mapping.  The array's address is looked up once per device
 * on the first call there (make that call outside graph capture).  Every call
 * on a device uses that device's one array: calls that overlap in time on one
 * device (other streams, other host threads) race and must be ordered by the
 * caller. */
#define PICASSO_STATIC_MAX_CLUSTERS (1 << 22)
int picasso_replace_mapping_static(int device, void* stream, const int32_t* d_cluster_id, int32_t n_in, int32_t n_out,
                                   int32_t* d_replace, int32_t* d_mapping, int32_t* d_status);

/* Member lists of the clusters: d_offsets [n_out+1], d_members [n_in] (members of
 * cluster c = d_members[d_offsets[c] .. d_offsets[c+1]), ascending).  Built with a
 * stable radix sort of (cluster_id, vertex).  Waits for its work on the stream (as
 * the decimate calls do); returns
 * PICASSO_ERR_BAD_INDEX if an id lies outside [0, n_out).  n_in <= 3*max_facets
 * and n_out <= max_verts of the context. */
int picasso_cluster_csr(picasso_ctx* ctx, void* stream, const int32_t* d_cluster_id, int32_t n_in, int32_t n_out,
                        int32_t* d_offsets, int32_t* d_members);

/* d_y [n_out, C] = pooled features.  d_weight [n_in] for PICASSO_POOL_WEIGHTED,
 * else may be NULL.  d_argmax [n_out, C] (vertex index, -1 for an empty cluster)
 * is written for PICASSO_POOL_MAX when not NULL.  Asynchronous on `stream`. */
int picasso_pool_forward(picasso_ctx* ctx, void* stream, int mode, const float* d_x, int32_t n_in, int32_t C,
                         const int32_t* d_offsets, const int32_t* d_members, int32_t n_out, const float* d_weight,
                         float* d_y, int32_t* d_argmax);

/* d_gx [n_in, C] = gradient with respect to the input features given d_gy
 * [n_out, C] (the adjoint of the forward pass; weights are constants).
 * PICASSO_POOL_MAX needs the d_argmax of the forward pass.  Asynchronous. */
int picasso_pool_backward(picasso_ctx* ctx, void* stream, int mode, const float* d_gy, int32_t n_in, int32_t C,
                          const int32_t* d_cluster_id, const int32_t* d_offsets, const int32_t* d_members,
                          int32_t n_out, const float* d_weight, const int32_t* d_argmax, float* d_gx);

/* Unpooling: d_x [n_in, C]: every vertex takes the feature of its cluster
 * (d_y [n_out, C]).  Its backward pass adds up the gradients of a cluster's
 * vertices (= PICASSO_POOL_SUM).  Asynchronous. */
int picasso_unpool_forward(picasso_ctx* ctx, void* stream, const float* d_y, int32_t n_in, int32_t C,
                           const int32_t* d_cluster_id, float* d_x);
int picasso_unpool_backward(picasso_ctx* ctx, void* stream, const float* d_gx, int32_t n_in, int32_t C,
                            const int32_t* d_offsets, const int32_t* d_members, int32_t n_out, float* d_gy);

/* ---- single steps of the path, exported for stage-level parity tests ------- */

/* Vertex quadrics (supplementary, facet and vertex quadric equations):
 * d_quadrics_out [N,10] = a00 a01 a02 a11 a12 a22 b0 b1 b2 c, each the
 * left-to-right fp32 sum over adjacent facets in ascending facet order
 * (vertex->facet lists by a sort of packed (vertex, facet) keys, then an
 * ordered segmented reduction).  Waits for its work on the stream. */
int picasso_vertex_quadrics(picasso_ctx* ctx, void* stream, const float* d_verts, int32_t N, const int32_t* d_facets,
                            int32_t F, float* d_quadrics_out);

/* Distinct edges of the input mesh in ascending (lo,hi) order (Alg. 2 line 1)
 * and the cost of each (Alg. 2 line 2) from the vertex quadrics above.
 * d_edges_out (capacity 3F*2 ints), d_cost_out (capacity 3F floats); the number
 * of edges goes to the host scalar h_ne_out.  Waits for its work on the stream. */
int picasso_edge_costs(picasso_ctx* ctx, void* stream, const float* d_verts, int32_t N, const int32_t* d_facets,
                       int32_t F, int32_t* d_edges_out, float* d_cost_out, int32_t* h_ne_out);

/* Plain device-to-device streaming copy kernel (16-byte accesses; nbytes and
 * both pointers multiples of 16).  Asynchronous on `stream`.  Used by the
 * benchmark as the HBM yardstick and to calibrate profiler byte counters. */
int picasso_device_copy(void* stream, void* d_dst, const void* d_src, size_t nbytes);

/* Stable LSD radix sort of n keys on their low `key_bits` bits, in place.
 * key_bytes is 4 or 8; d_vals (uint32, may be NULL) is permuted alongside.
 * n must not exceed 3*max_facets of the context. */
int picasso_radix_sort(picasso_ctx* ctx, void* stream, int key_bytes, void* d_keys, uint32_t* d_vals, int64_t n,
                       int key_bits);

/* Same contract as picasso_radix_sort, by the two-sweep method the path uses for
 * keys led by vertex ids: a partition on the top 8 of the key_bits, then one
 * workgroup per bucket sorts it in LDS (a bucket too large for LDS takes a slow
 * global-memory route).  2^20 < n <= 2^23 uses 4096 buckets on the top 12 bits
 * (needs key_bits > 12).  With values the partition is ordered (stable: per-tile
 * counts, row scans, ordered scatter; two 6-bit passes for 12 bits); without
 * values it is a single unordered pass, equal keys being indistinguishable. */
int picasso_bucket_sort(picasso_ctx* ctx, void* stream, int key_bytes, void* d_keys, uint32_t* d_vals, int64_t n,
                        int key_bits);

/* ---------------------------------------------------------------------------
 * Mesh convolutions, depth-wise form (Sec. 4 "Mesh Convolution"; supplementary
 * section "Backward propagations of different convolutions").  One filter
 * weight per channel; the channel-wise (dense) half of the paper's separable
 * convolutions is an ordinary matrix product and is left to the caller.
 * Features are fp32 row-major [rows, C]; all data pointers are device memory
 * owned by the caller.  Unless noted the calls are asynchronous on `stream`,
 * allocate nothing and do not report bad indices (an out-of-range index is read
 * as index 0): picasso_vertex_corner_csr checks a facet array once.  Any C >= 1.
 * ------------------------------------------------------------------------- */

/* Corners of the facet array at every vertex: corner i = 3 f + s is vertex
 * d_facets[i]; corners of vertex v = d_corners[d_offsets[v] .. d_offsets[v+1]),
 * ascending, so |N(v)| = d_offsets[v+1] - d_offsets[v] (a facet counts once per
 * corner).  d_offsets [N+1], d_corners [3F].  Waits for its work on the stream (as
 * the decimate calls do); returns
 * PICASSO_ERR_BAD_INDEX if an index lies outside [0, N).  F <= max_facets. */
int picasso_vertex_corner_csr(picasso_ctx* ctx, void* stream, const int32_t* d_facets, int32_t F, int32_t N,
                              int32_t* d_offsets, int32_t* d_corners);

/* Unit normals d_normals [F,3], areas d_areas [F] (Sec. 4, first paragraph; a
 * facet of zero area gets the zero normal) and interpolation levels d_level [F]
 * (Eq. "interpolate_num": k = floor((A - A_min) / (A_max - A_min)) * alpha +
 * beta, A_min and A_max over the facet's own mesh; the ratio counts as 0 when
 * all areas of a mesh are equal).  Any of the three outputs may be NULL.  B
 * meshes with h_nf[b] facets each (host array; NULL allowed for B = 1).
 * Waits for its work on the stream; PICASSO_ERR_BAD_INDEX as above. */
int picasso_facet_geometry(picasso_ctx* ctx, void* stream, const float* d_verts, int32_t N, const int32_t* d_facets,
                           int32_t F, int32_t B, const int32_t* h_nf, int32_t alpha, int32_t beta, float* d_normals,
                           float* d_areas, int32_t* d_level);

/* Fuzzy coefficients of the facets (Sec. 4.2): z_ft = |n_f - mu_t|^2 *
 * d_inv_var[t] (homogeneous diagonal covariance, inv_var = 1 / sigma_t^2),
 * pi_ft = exp(-z_ft) / sum_m exp(-z_fm).  d_normals [F,3], d_mu [T,3],
 * d_inv_var [T], d_pi [F,T]. */
int picasso_fuzzy_coefficients(picasso_ctx* ctx, void* stream, const float* d_normals, int32_t F, const float* d_mu,
                               const float* d_inv_var, int32_t T, float* d_pi);

/* Vertex2facet (Sec. 4.1): per channel J_f = (1/K) sum_k W_k I_k with I_k, W_k the
 * barycentric interpolations of the three vertex features and of the three
 * filter weights d_w [3,C] at the K = k (k + 1) / 2 points of level k =
 * d_level[f] (NULL: level 1 everywhere).  The points are the triangular lattice
 * (i, j, l) / (k - 1), i + j + l = k - 1 (the paper does not print them); level 1
 * is the centroid alone.  d_x [N,C] -> d_y [F,C]. */
int picasso_v2f_forward(picasso_ctx* ctx, void* stream, const float* d_x, int32_t N, int32_t C,
                        const int32_t* d_facets, int32_t F, const int32_t* d_level, const float* d_w, float* d_y);

/* Its backward pass (supplementary, vertex2facet kernel): d_gx [N,C] = gradient
 * with respect to the vertex features, d_gw [3,C] with respect to the filter;
 * either may be NULL.  d_offsets / d_corners from picasso_vertex_corner_csr of
 * the same facet array.  d_gw uses the context's workspace: calls on one
 * context that overlap in time race. */
int picasso_v2f_backward(picasso_ctx* ctx, void* stream, const float* d_gy, const float* d_x, int32_t N, int32_t C,
                         const int32_t* d_facets, int32_t F, const int32_t* d_level, const float* d_w,
                         const int32_t* d_offsets, const int32_t* d_corners, float* d_gx, float* d_gw);

/* Facet2facet (Sec. 4.1, for meshes rendered with textures): facet f carries the
 * texture points d_poff[f] .. d_poff[f+1] (d_poff [F+1], P points in all) with
 * features d_tex [P,C] and barycentric coordinates d_bary [P,3] that come with
 * the rendering; only the filter d_w [3,C] is interpolated, W_k = sum_s xi_ks w_s,
 * and J_f = (1 / Gamma_f) sum_k W_k T_k per channel (0 for a facet without
 * points).  d_y [F,C].  Offsets outside [0, P] are clipped. */
int picasso_f2f_forward(picasso_ctx* ctx, void* stream, const float* d_tex, const float* d_bary,
                        const int32_t* d_poff, int32_t F, int32_t P, int32_t C, const float* d_w, float* d_y);

/* Its backward pass (the supplementary refers to the vertex2facet kernel for it):
 * d_gtex [P,C] with respect to the texture features (rows of points that belong
 * to no facet are left untouched), d_gw [3,C] with respect to the filter; either
 * may be NULL.  d_gw uses the context's workspace as above. */
int picasso_f2f_backward(picasso_ctx* ctx, void* stream, const float* d_gy, const float* d_tex, const float* d_bary,
                         const int32_t* d_poff, int32_t F, int32_t P, int32_t C, const float* d_w, float* d_gtex,
                         float* d_gw);

/* Facet2vertex (Sec. 4.2, last equation): per channel I_v = (1 / |N(v)|) sum over the
 * corners at v of (sum_t pi_ft w_t) J_f; a vertex without facets gets 0.
 * d_y [F,C], d_pi [F,T], d_w [T,C] -> d_x [N,C]. */
int picasso_f2v_forward(picasso_ctx* ctx, void* stream, const float* d_y, int32_t F, int32_t C, const float* d_pi,
                        int32_t T, const float* d_w, const int32_t* d_offsets, const int32_t* d_corners, int32_t N,
                        float* d_x);

/* Its backward pass (supplementary, facet2vertex kernel): d_gy [F,C] with respect
 * to the facet features, d_gw [T,C] to the filter, d_gpi [F,T] to the fuzzy
 * coefficients (for learnable covariances); each may be NULL.  d_gw uses the
 * context's workspace as above. */
int picasso_f2v_backward(picasso_ctx* ctx, void* stream, const float* d_gx, const float* d_y, int32_t F, int32_t C,
                         const float* d_pi, int32_t T, const float* d_w, const int32_t* d_facets,
                         const int32_t* d_offsets, int32_t N, float* d_gy, float* d_gw, float* d_gpi);

#ifdef __cplusplus
}
#endif
#endif /* PICASSO_H */
