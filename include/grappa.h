/*
 * grappa.h - C ABI of the MI355X (gfx950) hot path of gradient-only GNN training:
 * the isolated per-partition train step and the coverage-corrected aggregation of
 * the partition gradients (Grappa, sections "Isolated Training Strategy",
 * "Coverage-Corrected Aggregation" and "Phase-Parallel Training").
 *
 * One iteration of the paper's phase-parallel algorithm with one partition active
 * at a time is, per partition p = 0..K-1:
 *     (isolated sampling) -> forward -> backward            grp_train_step
 *     scale grad by the coverage factor, reduce over p      grp_aggregate
 *     theta <- optimizer_step(theta, grad)                   grp_optimizer_step
 * on a local subgraph built once per (graph, K, seed, p) by grp_partition.
 *
 * General conventions
 *   - Pointers marked DEV are device (HBM) addresses, HOST are host addresses.  The
 *     caller owns every buffer it passes; the library owns only the opaque handles it
 *     returns and frees them in *_destroy.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls are
 *     asynchronous on that stream and do not synchronise it unless stated otherwise
 *     (the builders grp_partition*, grp_chunks_build*, grp_epoch_seeds and the inspection calls do;
 *     grp_train_step does not, in either mode).
 *   - Every function returns GRP_OK (0) or a negative status; it never throws or aborts.
 *     grp_last_error() gives a thread-local, library-owned description of the last
 *     failure on the calling thread.
 *   - Matrices are dense row-major; `ld*` is the row pitch in elements.  Values are expected to be finite: an
 *     infinity in a gathered feature row may come out as NaN (some kernels drop a row with a multiplication by 0).
 *   - Local node ids are int32, edge offsets int64 (a partition may hold 2^32 edges).
 */
#ifndef GRAPPA_H_
#define GRAPPA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t grp_status;
#define GRP_OK            0
#define GRP_EINVAL       (-1)   /* null pointer, K < 1, part_id outside [0,K), dims <= 0, ... */
#define GRP_ERANGE       (-2)   /* node id outside [0,N), local node count >= 2^31            */
#define GRP_ENOMEM       (-3)   /* a device allocation owned by a handle failed               */
#define GRP_EWORKSPACE   (-4)   /* caller's workspace is smaller than the queried size        */
#define GRP_EHIP         (-5)   /* a HIP runtime call failed (message has the HIP error)      */
#define GRP_EUNSUPPORTED (-6)   /* a combination this build does not implement                */

const char* grp_last_error(void);

/* ------------------------------------------------------------------ partition */

typedef struct grp_partition_s grp_partition_t;

/* Borrowed DEV pointers into a partition handle, valid until grp_partition_destroy.
 * CSR: row v lists the local sources u of the kept edges u->v, ascending; CSC: row u
 * lists the destinations, ascending.  Duplicate edges and self-loops are kept.       */
typedef struct {
    int64_t        n;            /* local nodes                                  */
    int64_t        nnz;          /* local edges (both endpoints owned)           */
    const int64_t* l2g;          /* [n]   global id of local node, ascending     */
    const int64_t* rowptr;       /* [n+1] CSR by destination                     */
    const int32_t* col;          /* [nnz] source local ids                       */
    const int64_t* colptr;       /* [n+1] CSC by source                          */
    const int32_t* row;          /* [nnz] destination local ids                  */
    const int32_t* d_local_in;   /* [n]   in-degree inside the partition         */
    const int32_t* d_local_out;  /* [n]   out-degree inside the partition        */
    const int64_t* d_global_in;  /* [n]   in-degree in the whole graph           */
} grp_partition_view_t;

/* Random node assignment and the isolated local subgraph ("Graph Partitioning": nodes
 * are assigned to partitions at random; "Isolated Training": only local nodes and
 * edges take part; no halo nodes: an edge with an endpoint in another partition is
 * dropped).
 *   owner(v) = SplitMix64_output(seed, v) mod K, where output number v (from 0) of the
 *   SplitMix64 sequence is mix(seed + (v+1)*0x9E3779B97F4A7C15) in wrapping uint64
 *   arithmetic, mix(z): z=(z^(z>>30))*0xBF58476D1CE4E5B9; z=(z^(z>>27))*0x94D049BB133111EB;
 *   z^(z>>31); the modulo is unsigned.
 * src/dst: DEV int64[E] global ids, edge e means dst[e] aggregates from src[e].
 * Degrees are in-degrees with multiplicity.  Local ids follow ascending global id.
 * Synchronous: returns after the handle is complete (it needs n and nnz on the host).
 * Errors: GRP_EINVAL (null, K<1, part_id, E<0, N<0), GRP_ERANGE (an id outside [0,N), or
 * n >= 2^31), GRP_ENOMEM, GRP_EHIP.  On error *out is NULL.                            */
grp_status grp_partition(const int64_t* src, const int64_t* dst, int64_t E, int64_t N,
                         int32_t K, uint64_t seed, int32_t part_id, void* stream,
                         grp_partition_t** out);

/* The node assignment alone: owner_out[v] = owner(v) for v in [0, N) (DEV int32[N]) and, if
 * count_out is not NULL, the number of nodes of every partition (DEV int64[K], overwritten).
 * Asynchronous on the stream.  Errors: GRP_EINVAL (N < 0, K < 1, null output), GRP_EHIP.      */
grp_status grp_node_owners(int64_t N, int32_t K, uint64_t seed, int32_t* owner_out,
                           int64_t* count_out, void* stream);

/* The same partition for neighbours of unequal weight (the general form of the coverage-corrected
 * estimators: a target distribution p_v(u) over the in-neighbours of v and a local one
 * q_v(u) = p_v(u) / sum of p_v over the local neighbours).  w: DEV float[E], w[e] > 0 finite, the
 * weight of edge e; p_v(u) = w(u->v) / (sum of the weights of all in-edges of v).  The handle then
 * also holds, readable through grp_partition_weights:
 *   csr_w / csc_w   DEV float[nnz]  the kept edges' weights in CSR / CSC order; equal (dst, src)
 *                                   pairs keep their order in the edge list
 *   w_local_in      DEV double[n]   sum of a node's local in-edge weights, added in CSR order
 *   w_global_in     DEV double[n]   sum over all its in-edges, added in edge-list order
 *                   (rows of more than 1024 weights: 256 consecutive runs added in order, then the
 *                   run sums added in order)
 * (both sums are sequential fp64 additions in the stated order, so they are reproducible bit
 * for bit).  grp_train_step on such a handle (GraphSAGE, full-graph mode; GRP_EUNSUPPORTED
 * otherwise) aggregates with the weighted mean m_v = sum_u w_uv h_u / w_local_in(v), and its
 * statistics use the weight masses: ratio = w_local_in / w_global_in (1 if w_global_in = 0),
 * R = sum_{v in S} (w_global_in - w_local_in) d_local / w_local_in (d_global for d_local = 0).
 * Errors as grp_partition, plus GRP_EINVAL for a weight that is not a positive finite number. */
grp_status grp_partition_weighted(const int64_t* src, const int64_t* dst, const float* w, int64_t E,
                                  int64_t N, int32_t K, uint64_t seed, int32_t part_id, void* stream,
                                  grp_partition_t** out);

typedef struct {
    const float*  csr_w;
    const float*  csc_w;
    const double* w_local_in;
    const double* w_global_in;
} grp_partition_weights_t;

/* Borrowed DEV pointers (all NULL for a partition built without weights). */
grp_status grp_partition_weights(const grp_partition_t* part, grp_partition_weights_t* view);

/* ------------------------------------------------------------------ chunks and sweeping partitions */

typedef struct grp_chunks_s grp_chunks_t;

/* The graph split once into chunks ("Chunks and Efficient Partition Construction"):
 *   chunk(v) = owner(v) of grp_partition with K = n_chunks (a random split).
 * The handle keeps a copy of the edge list grouped by (chunk(dst), chunk(src)) and every
 * node's global in-degree, so that a partition is later built from its own edges only.
 * src/dst: DEV int64[E] global ids.  1 <= n_chunks <= 64.  Synchronous.
 * Errors: GRP_EINVAL, GRP_ERANGE (an id outside [0,N)), GRP_ENOMEM, GRP_EHIP.              */
grp_status grp_chunks_build(const int64_t* src, const int64_t* dst, int64_t E, int64_t N,
                            int32_t n_chunks, uint64_t seed, void* stream, grp_chunks_t** out);
/* The same with the chunk of every node given by the caller instead of the random split, e.g. the
 * output of METIS or any other partitioner run beforehand ("Chunks and Efficient Partition
 * Construction": chunks come from unmodified partitioning strategies such as random or METIS).
 * chunk_of_node: DEV int32[N], values in [0, n_chunks); the handle keeps a copy.
 * Errors as grp_chunks_build, plus GRP_ERANGE for an assignment outside [0, n_chunks).          */
grp_status grp_chunks_build_assigned(const int64_t* src, const int64_t* dst, int64_t E, int64_t N,
                                     int32_t n_chunks, const int32_t* chunk_of_node, void* stream,
                                     grp_chunks_t** out);
grp_status grp_chunks_destroy(grp_chunks_t* chunks);

/* The training partition of a super-epoch: base chunk + swept chunk (swept == base: the base
 * chunk alone, which is grp_partition's partition `base` of K = n_chunks).  Nodes = the union
 * of the two chunks in ascending global id; edges = those with both endpoints in the union;
 * d_global_in = in-degree in the whole graph.  Same canonical CSR/CSC and the same handle as
 * grp_partition; only the edges of the four chunk pairs involved are read.  Worker i sweeps
 * chunk (i + 1 + t) mod n_chunks in super-epoch t (coverage guarantee paragraph: after
 * n_chunks - 1 super-epochs every pair of chunks has shared a partition).  Synchronous.     */
grp_status grp_partition_from_chunks(const grp_chunks_t* chunks, int32_t base, int32_t swept,
                                     void* stream, grp_partition_t** out);

/* Partition part_id extended by `hops` hops of read-only halo nodes ("Graph Partitioning":
 * an endpoint of a partition's edge that is not part of the partition is incorporated as a
 * halo node).  Hop 0 = the owned nodes; hop h adds the sources of every edge whose destination
 * lies in hops 0..h-1; the local edges are those whose destination lies in hops 0..hops-1, so
 * the outermost halo nodes carry features but no in-edges.  Local ids follow ascending global
 * id over the whole set; the owned nodes (the only loss nodes) are marked in the mask returned
 * by grp_partition_base_mask.  With hops >= the number of layers, a GraphSAGE or GAT step over
 * the owned nodes equals the whole-graph step restricted to them (d_local = d_global, c = 1).
 * 1 <= hops <= GRP_MAX_LAYERS (hops = 0 is grp_partition).  Same handle, same errors.       */
grp_status grp_partition_halo(const int64_t* src, const int64_t* dst, int64_t E, int64_t N,
                              int32_t K, uint64_t seed, int32_t part_id, int32_t hops,
                              void* stream, grp_partition_t** out);

/* DEV uint8[n]: 1 for the nodes of the base chunk (a partition's loss nodes are the training
 * nodes of its base chunk; the swept chunk only supplies neighbours), or for the owned nodes of
 * a halo partition.  *mask is NULL for partitions built by grp_partition / from a local COO.
 * Borrowed pointer, valid until the handle is destroyed.                                      */
grp_status grp_partition_base_mask(const grp_partition_t* part, const uint8_t** mask);

/* Adopt a partition's share that was generated directly as local edges.
 * src_local/dst_local: DEV int64[E] ids in [0,n).  d_global_in: DEV int64[n] or NULL
 * (= local in-degree, i.e. full coverage).  l2g: DEV int64[n] or NULL (= identity).
 * Builds the same canonical CSR/CSC as grp_partition.  Synchronous.                   */
grp_status grp_partition_from_local_coo(const int64_t* src_local, const int64_t* dst_local,
                                        int64_t E, int64_t n, const int64_t* d_global_in,
                                        const int64_t* l2g, void* stream, grp_partition_t** out);

/* Adopt a partition's share that already exists as rows of in-edges ("Isolated Training": a worker
 * holds exclusively its local nodes and edges; at the paper's largest scale, a trillion-edge graph
 * trained one partition at a time, a share has 2^32 edges, and an edge list of it plus the buffers of
 * a sort would not leave room for the step).
 *   rowptr  DEV int64[n+1]  0 = rowptr[0] <= ... <= rowptr[n] = nnz
 *   col     DEV int32[nnz]  local source ids in [0, n), ascending inside every row (duplicates kept)
 * The handle BORROWS both arrays: they are not copied, must stay valid and unchanged until
 * grp_partition_destroy, and are returned as they are by grp_partition_view.  The call builds the
 * transposed structure (colptr / row, destinations ascending), the degree arrays and the schedules of
 * the long rows; d_global_in / l2g as in grp_partition_from_local_coo (copied).
 *   slice_edges  upper bound on the edges transposed at a time (0 = 2^28): temporary device memory is
 *                about 24 bytes per edge of a slice; a slice holds whole runs of n/4096 consecutive
 *                sources, so the bound is raised to the largest such run if that is larger.
 * Synchronous.  Errors: GRP_EINVAL (null, negative sizes, row pointers that are not a non-decreasing
 * sequence from 0 to nnz, a row whose sources are not ascending), GRP_ERANGE (a source outside [0, n),
 * n >= 2^31), GRP_ENOMEM, GRP_EHIP.  On error *out is NULL.                                           */
grp_status grp_partition_from_csr(const int64_t* rowptr, const int32_t* col, int64_t n, int64_t nnz,
                                  const int64_t* d_global_in, const int64_t* l2g, int64_t slice_edges,
                                  void* stream, grp_partition_t** out);

grp_status grp_partition_view(const grp_partition_t* part, grp_partition_view_t* view /*HOST*/);
grp_status grp_partition_destroy(grp_partition_t* part);   /* NULL is a no-op */

/* ------------------------------------------------------------------ model */

#define GRP_MAX_LAYERS 16

#define GRP_ARCH_SAGE_MEAN    0  /* z_v = h_v W_self + mean_{u in N_v} h_u W_neigh + b        */
#define GRP_ARCH_GCN          1  /* z_v = sum_u Ahat[v,u] (h_u W) + b, symmetric normalisation */
#define GRP_ARCH_GCN_RESIDUAL 2  /* GCN with h^{l+1} = h^l + ReLU(z^l) where widths agree      */
#define GRP_ARCH_GAT          3  /* z_v = sum_u alpha_vu (h_u W) + b, attention weights alpha      */

#define GRP_DTYPE_FP32 0
#define GRP_DTYPE_BF16 1         /* storage of the input features only; accumulate in fp32 */

/* Model description (the paper's "GNN Models": GraphSAGE aggregates the neighbours'
 * states by averaging, combines with the node's own state and multiplies by a matrix;
 * GCN applies a linear map and averages neighbours with degree-based weights).
 * ReLU after every layer but the last; dropout is a step option (grp_step_opts).  GCN normalisation:
 * Ahat[v,u] = (A[v,u] + [u==v]) / sqrt((d_in(v)+1)(d_out(u)+1)) on local degrees when
 * gcn_self_loops != 0, else A[v,u] / sqrt(max(d_in(v),1) max(d_out(u),1)).
 * Flat parameter layout (weights in, gradients out): layer-major; per layer W_self
 * (GCN: W) row-major [dims[l] x dims[l+1]], then W_neigh (SAGE only), then b[dims[l+1]].
 * GAT (the third model of "GNN Models": the neighbours' states are combined with learned
 * attention weights; the published single-head layer): t = h W, score
 * e_vu = LeakyReLU_0.2(a_src . t_u + a_dst . t_v) over the in-edges u -> v (with
 * multiplicity) and one self term u = v, alpha = softmax_u(e_vu); full-graph mode only;
 * per-layer parameters W [dims[l] x dims[l+1]], a_src, a_dst, b (each [dims[l+1]]).        */
typedef struct {
    int32_t arch;
    int32_t n_layers;
    int32_t dims[GRP_MAX_LAYERS + 1];
    int32_t feat_dtype;
    int32_t gcn_self_loops;
} grp_model_desc;

/* Number of floats in the flat parameter vector, or -1 for an invalid description. */
int64_t grp_param_count(const grp_model_desc* model);

/* ------------------------------------------------------------------ train step */

#define GRP_EST_NONE           0  /* c = 1 (the paper's "no correction" ablation)             */
#define GRP_EST_NODE_LEVEL     1  /* asymptotically unbiased node-level estimator, uniform
                                     neighbours: node v's loss is weighted d_local/d_global   */
#define GRP_EST_BATCH_MIN_DIST 2  /* batch-level factor c = mean_v d_local/d_global           */
#define GRP_EST_SHRINKAGE      3  /* c = 1 / sum_v (d_global/d_local - 1)|S_v|                */

typedef struct {
    int32_t        estimator;     /* only NODE_LEVEL changes the step (per-node loss weights)  */
    int32_t        full_graph;    /* 1: whole partition each step; 0: mini-batch               */
    int32_t        n_seeds;       /* mini-batch: number of seed nodes                          */
    int32_t        reserved;
    const int32_t* seeds;         /* DEV int32[n_seeds] distinct local ids (mini-batch)        */
    int32_t        fanouts[GRP_MAX_LAYERS]; /* fanouts[l] belongs to layer l, 0 = input side   */
    uint64_t       sampler_seed;
    uint64_t       batch_id;
    float          dropout_rate;  /* in [0, 1); 0 = off (see below)                            */
    int32_t        flags;         /* GRP_STEP_* bits, 0 = defaults                              */
    uint64_t       dropout_seed;
    const uint64_t* batch_id_dev; /* DEV or NULL.  When set, batch_id above is ignored and the batch
                                     id (of the sampler and of dropout) is read from this address
                                     when the step's kernels run: a step captured in a HIP graph can
                                     then be replayed as the next batch by writing the new id (and the
                                     new seeds) into the same device buffers.                     */
} grp_step_opts;

/* grp_step_opts.flags.  A mini-batch step builds the transposed blocks (read by the backward pass only) on a
 * helper stream of the library's (default priority; one per caller stream, created at the first uncaptured
 * mini-batch step on that stream and kept) beside the next layers' sampling and the forward pass, and joins
 * it before the backward pass: shorter steps.  A caller that already runs several steps side by side on
 * streams of its own gains nothing from it and can keep every step on its one stream with this bit.     */
#define GRP_STEP_ONE_STREAM 1

/* Written to DEV memory by grp_train_step (one record per partition). */
typedef struct {
    double  loss;        /* (1/|S|) sum_{v in S} w_v (logsumexp z_v - z_v[y_v]); 0 if S empty */
    double  sum_ratio;   /* sum_{v in S} d_local(v)/d_global(v)  (1 if d_global = 0)          */
    double  R;           /* sum_{v in S} (d_global - d_local)|S_v|/d_local; full-graph:
                            sum (d_global - d_local), the number of dropped in-edges of S     */
    int64_t S;           /* nodes carrying loss                                               */
    int64_t nnz_used;    /* edges processed (local edges, or edges of the sampled blocks);
                            negative: minus the number of seeds outside the partition, the
                            record and the gradient of that step are invalid                  */
} grp_step_stats;

/* Bytes of caller-provided DEV workspace grp_train_step needs for this partition, model
 * and options (activations kept for the backward pass, temporaries, partial sums).     */
grp_status grp_step_workspace_bytes(const grp_partition_t* part, const grp_model_desc* model,
                                    const grp_step_opts* opts, size_t* bytes /*HOST*/);

/* One isolated train step on one partition (phase-parallel algorithm, the per-worker
 * body: isolated_sampling, forward_pass, backward_pass): loss and gradient of the mean
 * weighted softmax cross-entropy of the k-layer model over the loss nodes S, using only
 * the partition's local edges, plus the coverage statistics of S.
 *   features   DEV [n x dims[0]] row-major, fp32 or bf16 per model->feat_dtype
 *   labels     DEV int32[n], values in [0, dims[k])
 *   train_mask DEV uint8[n] or NULL (= all local nodes); full-graph mode only
 *   weights    DEV float[P] flat parameters (layout above)
 *   workspace  DEV, 256-byte aligned, at least the queried size; contents undefined after
 *   grad_out   DEV float[P], overwritten
 *   stats_out  DEV grp_step_stats, overwritten
 * S = train_mask ∩ local nodes (full graph) or the seeds (mini-batch).  Deterministic:
 * no floating-point atomics; two calls with equal inputs give equal bits.
 *
 * Dropout (the experimental setup trains with dropout 0.5; the paper fixes nothing else about it):
 * inverted dropout on the output of every layer but the last, after the ReLU (a residual layer
 * drops the activation before the skip is added): a' = keep ? a / (1 - rate) : 0, with
 *   key_l = mix(dropout_seed + (batch_id * GRP_MAX_LAYERS + l + 1) * 0x9E3779B97F4A7C15)
 *   keep(v, f) = (mix(key_l + (l2g[v] * dims[l+1] + f + 1) * 0x9E3779B97F4A7C15) >> 40)
 *                >= floor(dropout_rate * 2^24)
 * in wrapping uint64 arithmetic (mix as in grp_partition), so a node's mask depends on its global
 * id, not on the partition that holds it; 1 / (1 - rate) is taken in fp32.  The attention
 * coefficients of GRP_ARCH_GAT are not dropped.  In mini-batch mode v is the node a block row stands
 * for, and batch_id is the one the sampler uses.
 *
 * Mini-batch mode (opts->full_graph = 0, GraphSAGE only): isolated k-hop sampling inside the
 * partition, then the same layers on the sampled blocks.  Sampling rule (the paper fixes
 * none): per destination node v with d local in-edges all of them if d <= f = fanouts[l], else a
 * uniformly random f-subset of the positions 0..d-1 of v's CSR row, grown one element at a time:
 *   for t = 0..f-1:  top = d - f + t,  r = floor(u_t * (top + 1) / 2^64); the subset gains r if
 *   it does not hold r yet and top otherwise;
 *   u_t = M(M(M(M(M(sampler_seed) ^ batch_id) ^ l) ^ global_id(v)) ^ t),
 *   M(x) = SplitMix64 finaliser of x + 0x9E3779B97F4A7C15;
 * the chosen edges keep their row order; layers are built from the seeds inwards (the seeds draw
 * fanouts[k-1]); the mean
 * of a layer divides by the number of sampled neighbours.  Fanouts must lie in [1, 64]; seeds
 * must be distinct (not checked) and lie in [0, n).  This mode is as asynchronous as the full-graph
 * one: the sizes of the sampled blocks stay on the device, every launch is sized by the upper bounds
 * that follow from the seeds and fanouts (as is the workspace) and reads the real sizes from device
 * memory, so a step may be queued behind earlier work or captured in a HIP graph (no memset nodes are
 * recorded; a replay draws the same blocks unless the caller changes the seeds' contents, which are read
 * on the device).  The price is that an invalid seed list cannot fail the call: a seed outside [0, n)
 * is replaced by node 0 (no memory outside the partition is touched), and stats_out->nnz_used is set to
 * minus the number of such seeds; the other results of that step are then meaningless.
 * Errors: GRP_EINVAL, GRP_EWORKSPACE, GRP_EUNSUPPORTED (mini-batch with a GCN arch; a
 * residual first layer on bf16 features), GRP_EHIP.                                    */
grp_status grp_train_step(const grp_partition_t* part, const grp_model_desc* model,
                          const grp_step_opts* opts, const void* features,
                          const int32_t* labels, const uint8_t* train_mask,
                          const float* weights, void* workspace, size_t workspace_bytes,
                          void* stream, float* grad_out, grp_step_stats* stats_out);

/* Seed order of an epoch in mini-batch mode (the per-worker loop over batches of the phase-parallel
 * algorithm; the paper lets every worker visit all of its training nodes once per epoch and fixes no
 * order): the partition's training nodes (train_mask[v] != 0; NULL = every node; DEV uint8[n]) sorted
 * ascending by key(v) = M(M(M(sampler_seed) ^ epoch) ^ global_id(v)), M as in grp_train_step's sampling
 * rule, ties by local id.  seeds_out: DEV int32[n]; its first *n_seeds_out entries (HOST int64) are the
 * local ids in visiting order; batch b of size B is the slice [b*B, min((b+1)*B, *n_seeds_out)), to be
 * passed as opts->seeds / n_seeds.  Synchronous (the count is needed on the host); allocates and frees
 * O(n) temporary device memory.  Errors: GRP_EINVAL, GRP_ENOMEM, GRP_EHIP.                           */
grp_status grp_epoch_seeds(const grp_partition_t* part, const uint8_t* train_mask, uint64_t sampler_seed,
                           uint64_t epoch, void* stream, int32_t* seeds_out, int64_t* n_seeds_out /*HOST*/);

/* Inspection: where grp_train_step left the activation of layer `layer` inside the workspace it was
 * given (same partition, model and options).  *act_out is a borrowed DEV pointer into the workspace
 * to a [rows x *ld_out] row-major matrix (rows = n in full-graph mode; in mini-batch mode the layer's
 * destination nodes in block order: the seeds first, then each deeper layer's new nodes in ascending
 * local id) whose first dims[layer+1] columns hold
 * a_l = ReLU(z_l) of a hidden layer (after dropout if enabled, before a residual skip is added) or
 * the logits of the last layer; valid until the workspace is reused.  For callers that need the
 * ReLU decisions the step took (a checker comparing gradients with another implementation has to
 * take the same decision where a pre-activation is within rounding distance of zero).
 * Errors: GRP_EINVAL, GRP_EWORKSPACE.                                                            */
grp_status grp_step_activation(const grp_partition_t* part, const grp_model_desc* model,
                               const grp_step_opts* opts, void* workspace, size_t workspace_bytes,
                               int32_t layer, const float** act_out /*HOST*/, int64_t* ld_out /*HOST*/);

/* Inspection: the bipartite block that the isolated sampler of grp_train_step (mini-batch mode) built for
 * layer `layer` and left inside the workspace it was given (same partition, model and options;
 * "Isolated Training": k-hop subgraphs are sampled from the local partition only).  Borrowed DEV
 * pointers into the workspace, valid until it is reused:
 *   rowptr     int64[n_dst+1]  edges of destination row i: [rowptr[i], rowptr[i+1]), in ascending position
 *                              of the partition's CSR row
 *   col        int32[nnz]      layers >= 1: index into the block's source list; layer 0: partition-local id
 *   dst_nodes  int32[n_dst]    partition-local id of destination row i (the seeds for the last layer)
 *   src_nodes  int32[n_src]    layers >= 1: the block's source list = its destinations, then the newly
 *                              reached nodes in ascending local id; NULL for layer 0 (sources = all nodes)
 * Reads the block sizes back from the device: synchronises the device.
 * Errors: GRP_EINVAL (full-graph options, layer out of range), GRP_EWORKSPACE, GRP_EHIP.             */
typedef struct {
    int64_t        n_dst, n_src, nnz;
    const int64_t* rowptr;
    const int32_t* col;
    const int32_t* dst_nodes;
    const int32_t* src_nodes;
} grp_block_view_t;
grp_status grp_step_block(const grp_partition_t* part, const grp_model_desc* model, const grp_step_opts* opts,
                          void* workspace, size_t workspace_bytes, int32_t layer, grp_block_view_t* view /*HOST*/);

/* ------------------------------------------------------------------ aggregation */

/* Coverage-corrected aggregation ("Coverage-Corrected Aggregation"; the scale-then-
 * all_reduce lines of the phase-parallel algorithm):  G = (1/K) sum_p c_p g_p  with
 *   c_p = 1                                  NONE, NODE_LEVEL
 *   c_p = sum_ratio_p / S_p  (1 if S_p = 0)  BATCH_MIN_DIST   (uniform batch-level factor)
 *   c_p = 1 / R_p            (1 if R_p = 0)  SHRINKAGE        (shrinkage equation)
 *   grads   DEV float, partition p's gradient starts at grads + p*ld_grads, P floats
 *   stats   DEV grp_step_stats[K]
 *   update  DEV float[P], overwritten;  c_out DEV float[K] or NULL
 * Sums over p in ascending order with fp32 fused multiply-adds.  Errors: GRP_EINVAL.   */
grp_status grp_aggregate(const float* grads, int64_t ld_grads, const grp_step_stats* stats,
                         int32_t K, int64_t P, int32_t variant, void* stream,
                         float* update, float* c_out);
/* The same reduction over K separately owned gradient buffers (the buffers a framework's backward pass fills,
 * as the paper's gradient hook sees them): grads is a DEV array of K DEV pointers, each to P floats.
 * aligned16 != 0 promises that every buffer is 16-byte aligned (16-byte loads); results are the same bits either
 * way, and the same as grp_aggregate's on the same values.                                                  */
grp_status grp_aggregate_ptrs(const float* const* grads, int32_t aligned16, const grp_step_stats* stats,
                              int32_t K, int64_t P, int32_t variant, void* stream,
                              float* update, float* c_out);

/* ------------------------------------------------------------------ training controller (host arithmetic) */

/* The chunk worker `worker` (base chunk = worker) sweeps in super-epoch t: (worker + 1 + (t mod (c-1))) mod c for
 * c = n_chunks > 1, 0 for c = 1 (coverage guarantee paragraph: after c - 1 super-epochs every pair of chunks
 * has shared a partition; then the cycle repeats).  -1 for arguments out of range.                         */
int32_t grp_sweep_chunk(int32_t worker, int64_t super_epoch, int32_t n_chunks);
/* Epochs per super-epoch: ceil(e / (c - 1)) for e epochs in all ("Training Controller and Partitions Switching":
 * the e epochs are spread over the c - 1 super-epochs of a cycle), at least 1; -1 for arguments out of range. */
int64_t grp_super_epoch_epochs(int64_t total_epochs, int32_t n_chunks);

/* The controller (same subsection): it lets a super-epoch run its epochs and switches partitions earlier once
 * the coverage deficit of a step, 1 - mean over the step's active partitions of the minimum-distance factor
 * c_hat_p = sum_ratio_p / S_p (1 if S_p = 0), has exceeded `threshold` on `patience` consecutive steps (the paper
 * monitors the deficit and gives neither number: both are the caller's).  Host object; not thread-safe.   */
typedef struct grp_controller_s grp_controller_t;
grp_status grp_controller_create(int64_t total_epochs, int32_t n_chunks, double threshold, int64_t patience,
                                 grp_controller_t** out);
/* One training step: c_hat HOST float[m] (e.g. c_out of grp_aggregate with GRP_EST_BATCH_MIN_DIST), or the step's
 * statistics records themselves, HOST grp_step_stats[m] (a copy of what grp_train_step wrote), m >= 1.        */
grp_status grp_controller_observe(grp_controller_t* ctl, const float* c_hat, int32_t m);
grp_status grp_controller_observe_stats(grp_controller_t* ctl, const grp_step_stats* stats, int32_t m);
/* End of an epoch: *switched = 1 if the partitions must be rebuilt for the next super-epoch (its number is
 * then one higher and the step streak starts again).                                                        */
grp_status grp_controller_end_epoch(grp_controller_t* ctl, int32_t* switched /*HOST*/);
grp_status grp_controller_state(const grp_controller_t* ctl, int64_t* super_epoch /*HOST or NULL*/,
                                int64_t* epochs_per_super_epoch /*HOST or NULL*/);
grp_status grp_controller_destroy(grp_controller_t* ctl);   /* NULL is a no-op */

/* ------------------------------------------------------------------ optimizer */

#define GRP_OPT_SGD  0
#define GRP_OPT_ADAM 1

/* Hyper-parameters of the optimizer step.  The paper fixes only the learning rate (0.003,
 * experimental setup) and names no optimizer; ADAM is the published algorithm of Kingma &
 * Ba (bias-corrected moments, no weight decay), SGD is theta - lr * update.              */
typedef struct grp_optimizer_desc {
    int32_t kind;            /* GRP_OPT_SGD | GRP_OPT_ADAM                                  */
    int32_t reserved;
    float   lr;              /* > 0                                                         */
    float   beta1, beta2;    /* ADAM: in [0, 1)                                             */
    float   eps;             /* ADAM: > 0                                                   */
} grp_optimizer_desc;

/* theta <- optimizer_step(theta, update): the last line of an iteration of the phase-
 * parallel algorithm; theta and the optimizer state (m, v, the step count) are the
 * caller's and carry over from phase to phase.
 *   theta   DEV float[P], updated in place
 *   update  DEV float[P], the aggregated gradient G (read only)
 *   m, v    DEV float[P] first / second moment, updated in place (ADAM; ignored for SGD,
 *           may be NULL then); the caller zero-fills them before step 1
 *   step    1-based count of this step (ADAM's bias correction)
 * fp32 arithmetic, one pass over the arrays.  Errors: GRP_EINVAL (null pointer, P < 0,
 * step < 1, hyper-parameters out of range).                                              */
grp_status grp_optimizer_step(const grp_optimizer_desc* opt, int64_t P, int64_t step, float* theta,
                              const float* update, float* m, float* v, void* stream);

/* The rows of a partition out of a tensor indexed by global node id (the feature movement the paper
 * defers to repartitioning boundaries: when the partitions of a super-epoch are built, every worker
 * takes its nodes' rows of the feature / label / mask tensors): out[r, :] = src[idx[r], :] for r in
 * [0, n), rows of row_bytes bytes, both tensors dense row-major.
 *   src   DEV [n_src x row_bytes]      idx  DEV int64[n] (a partition's l2g)      out  DEV [n x row_bytes]
 *   keep  DEV uint8[n] or NULL: rows with keep[r] == 0 are zero-filled instead (e.g. the loss mask of a
 *         sweeping partition: the training mask of its base chunk's nodes only)
 * A row whose index is outside [0, n_src) is zero-filled.  16-byte moves when row_bytes and both
 * pointers allow it.  Asynchronous on the stream.  Errors: GRP_EINVAL, GRP_EHIP.                    */
grp_status grp_gather_rows(const void* src, int64_t n_src, int64_t row_bytes, const int64_t* idx, int64_t n,
                           const uint8_t* keep, void* out, void* stream);

/* ------------------------------------------------------------------ building blocks */

#define GRP_SCALE_NONE  0
#define GRP_SCALE_MEAN  1
#define GRP_SCALE_RSQRT 2
/* Neighbour aggregation on a partition (the message-passing step of every layer):
 *   transposed = 0:  Y[v,:] = a_v (sum_{u->v} X[u,:] + self*X[v,:])     rows of the CSR
 *   transposed = 1:  Y[u,:] = a_u (sum_{u->v} X[v,:] + self*X[u,:])     rows of the CSC
 * a = 1 (scale GRP_SCALE_NONE), 1/max(deg,1) (MEAN) or 1/sqrt(deg+self) clamped at
 * deg>=1 (RSQRT), deg = the row's length.  X: DEV [n x F] fp32/bf16, Y: DEV [n x F] fp32.
 * Scratch for the partial sums of the rows the partition splits (rows of more than 128 edges):
 * grp_spmm_workspace_bytes gives the size for this direction and F (0 when no row is split); `workspace`
 * is DEV, 16-byte aligned, contents undefined afterwards.  The call allocates nothing and is asynchronous
 * on the stream.  Errors: GRP_EINVAL, GRP_EWORKSPACE, GRP_EUNSUPPORTED (F > 1024).                    */
grp_status grp_spmm_workspace_bytes(const grp_partition_t* part, int32_t transposed, int32_t F, size_t* bytes /*HOST*/);
grp_status grp_spmm(const grp_partition_t* part, int32_t transposed, int32_t scale,
                    int32_t self_term, int32_t F, const void* X, int64_t ldx, int32_t x_dtype,
                    float* Y, int64_t ldy, void* workspace, size_t workspace_bytes, void* stream);

/* grp_spmm for callers that cannot allocate device memory or pass a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the partial sums of the split rows live
 * in a scratch array built into the library, 32 MiB per GPU, reserved when the library is loaded and kept
 * until the process ends.  Same arguments, kernels and results (bit for bit) as grp_spmm.  A partition
 * whose split rows need more than 32 MiB at this F (more than 32 MiB / (4 * round_up(F, 4)) chunks of 512
 * edges) is refused with GRP_EWORKSPACE; nothing is allocated or freed.  All calls on one GPU share that
 * GPU's array: calls that may overlap in time on one GPU (different streams or threads) race on it and
 * must be serialised by the caller; calls on one stream are safe.                                      */
grp_status grp_spmm_static(const grp_partition_t* part, int32_t transposed, int32_t scale,
                           int32_t self_term, int32_t F, const void* X, int64_t ldx, int32_t x_dtype,
                           float* Y, int64_t ldy, void* stream);

/* Dense transforms on the matrix cores (fp32 MFMA, fp32 accumulate):
 *   grp_gemm_nn:  C[M x N] = A[M x K] B[K x N]            (X W, dY W^T with B given transposed)
 *   grp_gemm_tn:  C[K x N] = A[M x K]^T B[M x N]          (X^T dY), reduction over M in a
 *                 fixed order; `workspace` DEV of grp_gemm_tn_workspace_bytes(M,K,N).   */
grp_status grp_gemm_nn(int64_t M, int32_t N, int32_t K, const void* A, int64_t lda,
                       int32_t a_dtype, const float* B, int64_t ldb, float* C, int64_t ldc,
                       void* stream);
/*   grp_gemm_nt:  C[M x N] = A[M x K] Bt[N x K]^T         (B given transposed, k contiguous: the
 *                 layout the train step keeps its weights in; fastest path)               */
grp_status grp_gemm_nt(int64_t M, int32_t N, int32_t K, const void* A, int64_t lda,
                       int32_t a_dtype, const float* Bt, int64_t ldbt, float* C, int64_t ldc,
                       void* stream);
size_t     grp_gemm_tn_workspace_bytes(int64_t M, int32_t K, int32_t N);
grp_status grp_gemm_tn(int64_t M, int32_t K, int32_t N, const void* A, int64_t lda,
                       int32_t a_dtype, const float* B, int64_t ldb, float* C, int64_t ldc,
                       void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------ tuning */

/* Which partitions also get the source-sliced schedule of their long rows when they are built: those with at
 * least min_nodes nodes (default 2^19) whose rows of more than 128 edges hold at least min_long_edge_percent
 * of the edges of that direction (default 25).  Below either bound the partial rows cost more than the cache hits save (a 3·10^5-node share whose
 * feature matrix about fits the last-level cache: 5 % slower aggregation with the schedule).  Such rows are cut where their sorted sources
 * pass from one of 64 equal ranges of node ids into the next, and the aggregation then processes the pieces
 * range by range, so that the rows gathered at any one time come from one 64th of the nodes and stay in the L2
 * cache.  Results differ from the unsliced schedule only by the order of fp32 additions (both orders are fixed
 * by the graph).  Applies to partitions built afterwards; process-wide.  min_nodes >= 1, percent in [0, 100]. */
grp_status grp_set_slice_policy(int64_t min_nodes, int32_t min_long_edge_percent);

/* ------------------------------------------------------------------ profiling */

/* Per-kernel timing with HIP events on the launch stream.  While enabled, every kernel
 * the library launches is bracketed by two events.  grp_profile_report synchronises the
 * recorded events, writes one line "name launches total_ms total_flops total_bytes\n"
 * per kernel name into buf (HOST, NUL-terminated, truncated to cap) and clears the
 * records.  flops/bytes are the algorithmic work of the launches (operand and result
 * sizes, 2*M*N*K), not measured traffic.                                              */
grp_status grp_profile_enable(int32_t on);   /* 0 off, 1 per kernel name, 2 names carry the launch shape */
grp_status grp_profile_report(char* buf, size_t cap);

#ifdef __cplusplus
}
#endif
#endif /* GRAPPA_H_ */
