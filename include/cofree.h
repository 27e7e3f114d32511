/*
 * cofree.h - C ABI of the MI355X (gfx950) hot path of communication-free vertex-cut GNN
 * training (arxiv 2308.03209): full-batch forward + backward of a GNN on ONE vertex-cut
 * partition, with Degree-Aware Reweighting of the loss and DropEdge-K masks.
 *
 * Conventions
 *  - Every function returns a cofree_status (0 = ok) unless stated; nothing throws across
 *    the boundary.  cofree_last_error() gives a thread-local message for the last failure.
 *  - "host" pointers are ordinary process memory; "device" pointers are HIP device memory of
 *    the current device.  The library never takes ownership of caller buffers.
 *  - The library owns only the opaque cofree_partition / cofree_masks objects (host copies of
 *    the graph arrays plus device copies made with hipMalloc); free them with the *_free calls.
 *  - All matrices are row-major and contiguous: element (r, c) of an [R, C] matrix is at r*C + c.
 *    Device matrices handed to the layer calls start at a 16-byte aligned address (COFREE_EINVAL if not).
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Layer, loss and
 *    step calls only enqueue kernels on it and never synchronise.
 *  - With COFREE_OVERLAP=1 in the environment cofree_layer_bwd runs part of its work on a second stream
 *    the library owns (one per device, default priority), forked from and joined back into `stream` by
 *    events inside the call; to the caller the call behaves as if everything ran on `stream`.  That
 *    stream and its events are shared by all calls on a device: issue layer calls for one device from
 *    one host thread at a time.  Without it (the default) everything is enqueued on `stream`.
 *  - More environment variables override launch choices that the library otherwise makes from the
 *    shapes; results are the same to rounding order, they exist for tuning and so that tests can send small
 *    inputs through every kernel: COFREE_AGG_SLICES = 0 | 1 | 8 (aggregation: row kernel, neighbour-group
 *    kernel, the same in 8 column slices), COFREE_AGG_BUCKETS = 0 (aggregation: no degree buckets - hub rows
 *    are not split over a workgroup and one kernel, chosen from the average degree, takes every row),
 *    COFREE_AGG_ENTRY_SCALE = 0 | 1 (aggregation: per-source factors gathered from the per-node vector, or read
 *    per adjacency entry next to the neighbour ids), COFREE_AGG_SLOTS = 0 (aggregation: the row kernel reads
 *    the graph by row id instead of walking the copy stored in processing order) and
 *    COFREE_BF16_TILE = 128 | 256 (block tile of the bfloat16 products C = A B^T).  All are read at every launch.
 *  - Parameters, gradients, norms, loss weights and the loss are float32.  Features and
 *    activations have the layer's dtype (COFREE_F32, or COFREE_BF16 with float32 accumulation).
 */
#ifndef COFREE_H
#define COFREE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum cofree_status {
  COFREE_OK = 0,
  COFREE_EINVAL = 1, /* bad argument (message says which) */
  COFREE_ENOMEM = 2, /* host or device allocation failed, or workspace too small */
  COFREE_EHIP = 3,   /* a HIP runtime call failed */
  COFREE_ESTATE = 4  /* object not in the required state (e.g. no device copy) */
} cofree_status;

typedef enum cofree_dtype { COFREE_F32 = 0, COFREE_BF16 = 1 } cofree_dtype;
typedef enum cofree_layer_kind { COFREE_GCN = 0, COFREE_SAGE_MEAN = 1, COFREE_SAGE_CONV = 2 } cofree_layer_kind;
typedef enum cofree_weight_kind {
  COFREE_W_DAR = 0,    /* Degree-Aware Reweighting, D(v_j[i]) / D(v_j) (Eq. 3) */
  COFREE_W_NONE = 1,   /* ones: every copy of a node counts fully (ablation of Section 5.3) */
  COFREE_W_CUSTOM = 2, /* caller's device vector */
  COFREE_W_INV_RF = 3  /* 1 / RF(v_j) (the "vanilla-inv" ablation); the partition must be built with COFREE_WITH_RF */
} cofree_weight_kind;
typedef enum cofree_step_kind { COFREE_SGD = 0, COFREE_ADAM = 1 } cofree_step_kind;

/* flags of cofree_build_partition */
#define COFREE_DEDUP 1u     /* drop repeated edges instead of rejecting them */
#define COFREE_HOST_ONLY 2u /* build host arrays only; no device copy (no GPU needed) */
#define COFREE_WITH_RF 4u   /* also count, per node, the partitions that hold a copy of it (Eq. 1 per node) */
#define COFREE_CUT_DBH 8u   /* degree-aware hash cut instead of the random cut (see cofree_build_partition) */

/* arrays of a partition, for cofree_partition_host_array / _device_array */
typedef enum cofree_array {
  COFREE_ARR_LOCAL2GLOBAL = 0, /* int64 [n_nodes]   duplicated-node map: global id of each local node, ascending */
  COFREE_ARR_ROWPTR = 1,       /* int64 [n_nodes+1] CSR row offsets */
  COFREE_ARR_COL = 2,          /* int32 [nnz]       neighbour local ids, ascending within a row */
  COFREE_ARR_EID = 3,          /* int32 [nnz]       undirected edge id of each CSR entry (host only) */
  COFREE_ARR_DEG_LOCAL = 4,    /* int32 [n_nodes]   D(v_j[i]): degree inside the partition, before masks */
  COFREE_ARR_DEG_GLOBAL = 5,   /* int32 [n_nodes]   D(v_j): degree in the full graph */
  COFREE_ARR_DAR_WEIGHT = 6,   /* float [n_nodes]   D(v_j[i]) / D(v_j) */
  COFREE_ARR_EDGE_LO = 7,      /* int32 [n_edges]   smaller local endpoint of undirected edge e (host only) */
  COFREE_ARR_EDGE_HI = 8,      /* int32 [n_edges]   larger local endpoint (host only) */
  COFREE_ARR_RF = 9            /* int32 [n_nodes]   RF(v_j): partitions holding the node (host only; COFREE_WITH_RF) */
} cofree_array;

typedef struct cofree_partition cofree_partition;
typedef struct cofree_masks cofree_masks;

const char* cofree_last_error(void);
/* Number of HIP devices visible, or -1 if the runtime cannot be initialised. Never faults. */
int32_t cofree_device_count(void);
/* sizeof(cofree_layer_desc) as the library was built with: a binding compares it with its own layout before
 * it passes descriptors across the boundary. */
size_t cofree_layer_desc_size(void);

/* ---------------------------------------------------------------------------------------
 * Vertex-cut partition (Section 3 "Vertex Cut Partitioning"; Algorithm 1 lines 1 and 4).
 *
 * Input: an undirected simple graph as n_edges (src[e], dst[e]) host pairs over node ids
 * 0..n_nodes-1 (n_nodes <= 2^32), each edge listed once in either orientation.  Self-loops
 * and out-of-range ids give COFREE_EINVAL; so do repeated edges unless COFREE_DEDUP is set (with an explicit
 * assignment repeats are always rejected: two copies could be sent to different partitions).
 * The edge set is split into n_parts disjoint subsets by the random vertex cut of the proof
 * of Theorem 2: edge {lo < hi} goes to partition floor(r * n_parts / 2^32), r = word 0 of
 * Philox-4x32-10 with counter (lo, hi, 0, 1) and key (seed mod 2^32, seed div 2^32) - or to
 * assignment[e] when `assignment` (host, int32[n_edges], values in [0, n_parts)) is given.
 * With COFREE_CUT_DBH the cut is degree-aware instead (Appendix A: cutting the higher-degree
 * vertices leaves fewer mirror vertices; the degree-based hashing compared in Appendix C): the
 * edge goes to floor(r * n_parts / 2^32), r = word 0 of Philox with counter (v, 0, 1, 1), v the
 * endpoint of smaller global degree (the smaller id on a tie), so only high-degree nodes are
 * replicated.
 * Partition `part_id` is built: V[i] = endpoints of E[i], numbered by ascending global id;
 * CSR with both directions of every edge and ascending neighbour ids (the graph is symmetric,
 * so the same arrays are its CSC); undirected edge ids = rank of (lo_local, hi_local);
 * degrees count distinct neighbours; Degree-Aware Reweighting weight of a node =
 * float(double(D_local) / double(D_global)) (Section 4.3).
 * Unless COFREE_HOST_ONLY is set the arrays the kernels need are copied to the current device.
 * *out is owned by the library until cofree_partition_free.
 */
int32_t cofree_build_partition(int64_t n_nodes, int64_t n_edges, const int64_t* src, const int64_t* dst,
                               int32_t n_parts, int32_t part_id, uint64_t seed, const int32_t* assignment,
                               uint32_t flags, cofree_partition** out);
void cofree_partition_free(cofree_partition* part);

/* The same partition from an edge list that arrives in pieces (Section 3 "Vertex Cut Partitioning"; Algorithm 1
 * lines 1 and 4), for graphs whose edge list does not fit host memory: the random cut decides every edge by
 * itself, so partition `part_id` only has to keep the edges that hash into it, while D(v) is counted for every
 * edge that passes.  Host memory: 4 bytes per node of the full graph plus the partition.
 *   _begin      flags: COFREE_DEDUP, COFREE_HOST_ONLY, COFREE_WITH_RF (COFREE_CUT_DBH gives COFREE_EINVAL: the
 *               degree-aware cut needs every degree before the first edge is assigned; no explicit assignment).
 *   _add_edges  n_edges host pairs as for cofree_build_partition; may be called any number of times.  Repeats
 *               inside one call are dropped with COFREE_DEDUP and rejected without it.  The caller guarantees
 *               that copies of one edge never arrive in different calls (for instance by streaming the edges
 *               grouped by one endpoint): such copies are detected by _finish only if they fall into this
 *               partition (COFREE_EINVAL); elsewhere they would be counted twice in D(v).
 *               A piece that is rejected with COFREE_EINVAL leaves the builder as it was; after COFREE_ENOMEM
 *               the piece may have been counted in part and the builder can only be freed.
 *   _finish     builds the partition exactly as cofree_build_partition does from the concatenated list (same
 *               arrays bit for bit), uploads it unless COFREE_HOST_ONLY, and frees the builder - also on error.
 *   _free       abandons a builder without finishing it.
 * One builder is fed from one host thread at a time. */
typedef struct cofree_partition_builder cofree_partition_builder;
int32_t cofree_partition_builder_begin(int64_t n_nodes, int32_t n_parts, int32_t part_id, uint64_t seed,
                                       uint32_t flags, cofree_partition_builder** out);
int32_t cofree_partition_builder_add_edges(cofree_partition_builder* builder, int64_t n_edges, const int64_t* src,
                                           const int64_t* dst);
int32_t cofree_partition_builder_finish(cofree_partition_builder* builder, cofree_partition** out);
void cofree_partition_builder_free(cofree_partition_builder* builder);

/* Replication factor of a cut (Eq. 1): RF = (1 / |V|) * sum_i |V[i]| over the n_parts partitions given (host
 * handles, all built from the same graph of n_nodes_full nodes).  Host-side, no device work. */
int32_t cofree_replication_factor(int64_t n_nodes_full, const cofree_partition* const* parts, int32_t n_parts,
                                  double* rf_out);
int64_t cofree_partition_num_nodes(const cofree_partition* part); /* |V[i]| */
int64_t cofree_partition_num_edges(const cofree_partition* part); /* |E[i]|, undirected */
int64_t cofree_partition_num_nnz(const cofree_partition* part);   /* 2 |E[i]| */
/* Read-only view of one array (see cofree_array); *count = number of elements. */
int32_t cofree_partition_host_array(const cofree_partition* part, int32_t which, const void** ptr, int64_t* count);
int32_t cofree_partition_device_array(const cofree_partition* part, int32_t which, const void** ptr, int64_t* count);

/* ---------------------------------------------------------------------------------------
 * DropEdge-K (Section 4.4; Algorithm 1 lines 5 and 7-9): K masks over E[i] drawn once.
 * Mask k keeps undirected edge e iff word 0 of Philox-4x32-10 with counter (e, 0, k, 2) and
 * key from `seed` is >= floor(p_drop * 2^32); 0 <= p_drop < 1, K >= 1.  The bits are drawn by
 * a HIP kernel; for each mask the kept edges are compacted into a CSR of their own, with the
 * masked degrees and normalisation vectors, and kept on the device.  The call synchronises.
 * The masked edge set is the graph of an iteration: means and GCN normalisation use masked
 * degrees; Degree-Aware Reweighting weights are unchanged by masks.
 */
int32_t cofree_dropedge_k(const cofree_partition* part, int32_t K, double p_drop, uint64_t seed, uint32_t flags,
                          void* stream, cofree_masks** out);
void cofree_masks_free(cofree_masks* masks);
int32_t cofree_masks_count(const cofree_masks* masks);
/* Host copy of mask k's bits: bit e%64 of word e/64 is 1 iff edge e is kept; *n_words = ceil(|E[i]|/64). */
int32_t cofree_masks_host_bits(const cofree_masks* masks, int32_t k, const uint64_t** words, int64_t* n_words);
/* Host copy of mask k's compacted CSR (rowptr int64[n_nodes+1], col int32[*nnz]). */
int32_t cofree_masks_host_graph(const cofree_masks* masks, int32_t k, const int64_t** rowptr, const int32_t** col,
                                int64_t* nnz);
/* Mask used by iteration `epoch` (Algorithm 1 line 8): floor(r * K / 2^32), r = word 0 of Philox
 * with counter (epoch mod 2^32, epoch div 2^32, 0, 3).  Host-side, no device work. */
int32_t cofree_dropedge_pick(uint64_t seed, uint64_t epoch, int32_t K, int32_t* k_out);

/* ---------------------------------------------------------------------------------------
 * Neighbour aggregation on the (masked) partition graph - the sparse kernel of the path.
 *   mode COFREE_AGG_MEAN      Y[v] = (1/deg v) * sum_{u in N(v)} X[u]            (0 if deg v = 0)
 *   mode COFREE_AGG_MEAN_T    Y[u] = sum_{v in N(u)} X[v] / deg v                (transpose of MEAN)
 *   mode COFREE_AGG_GCN       Y[v] = s_v * (s_v X[v] + sum_{u in N(v)} s_u X[u]), s = 1/sqrt(deg+1)
 * (the GCN matrix is symmetric, so it is its own transpose).  X, Y: device [n_nodes, width],
 * dtype as given, X != Y.  masks may be NULL (unmasked partition graph); else mask_id selects
 * the mask.  The transpose is a pull over the same symmetric CSR: no atomics.
 */
typedef enum cofree_agg_mode { COFREE_AGG_MEAN = 0, COFREE_AGG_MEAN_T = 1, COFREE_AGG_GCN = 2 } cofree_agg_mode;
int32_t cofree_aggregate(const cofree_partition* part, const cofree_masks* masks, int32_t mask_id, int32_t mode,
                         const void* X, void* Y, int32_t width, int32_t dtype, void* stream);

/* ---------------------------------------------------------------------------------------
 * One GNN layer on the partition (Section 3; Algorithm 1 line 10 evaluates L of them).
 *
 * COFREE_SAGE_MEAN - the GraphSAGE-mean layer as the paper prints it:
 *     h_v' = U . CONCAT( MEAN{ ReLU(W h_u + bW) : u in N(v) }, h_v ) + bU
 *   W [d_msg, d_in], bW [d_msg], U [d_out, d_msg + d_in] (message block first), bU [d_out].
 * COFREE_GCN - H' = act( S (A + I) S . H . W^T + bW ), S = diag(1/sqrt(deg+1)) on the partition
 *   graph; W [d_out, d_in], bW [d_out]; act = ReLU if desc.act != 0.  d_msg is ignored.
 * COFREE_SAGE_CONV - the conventional GraphSAGE-mean layer (the stock layer of the experiments,
 *   Section 5.1): h_v' = act( W_self h_v + W_neigh . MEAN{ h_u : u in N(v) } + bW );
 *   W [d_out, 2 d_in] = [W_self | W_neigh], bW [d_out]; act as for GCN; d_msg, U, bU are ignored.
 *   The mean commutes with W_neigh and is taken on min(d_in, d_out) columns.
 * N(v) and deg are those of the masked partition graph.  If dropout_q > 0 the layer output is
 * multiplied by keep/(1-q), keep(r,c) = [word (i%4) of Philox(counter (i/4 mod 2^32, i/4 div 2^32,
 * epoch mod 2^32, 4 + 256*layer_id), key seed) >= floor(q * 2^32)], i = r*d_out + c.
 */
typedef struct cofree_layer_desc {
  int32_t kind;  /* cofree_layer_kind */
  int32_t dtype; /* cofree_dtype of H_in, H_out and saved activations */
  int32_t d_in, d_msg, d_out;
  int32_t act;   /* GCN and SAGE_CONV: 1 = ReLU on the output, 0 = none */
  float dropout_q; /* 0 <= q < 1 */
  int32_t layer_id;
  uint64_t seed;  /* dropout seed */
  uint64_t epoch; /* iteration number (dropout counter) */
  uint32_t grad_flags; /* backward only, see below; 0 = plain gradients */
  float dropout_q_below; /* with COFREE_GRAD_IN_GATED: dropout rate q of the layer below, in [0, 1) */
} cofree_layer_desc;

/* grad_flags: the backward of a layer's ReLU and dropout (gradient zeroed where the output is not positive,
 * times 1/(1-q)) is an elementwise pass over [n_nodes, d_out]; between two stacked layers it can ride on the
 * kernel that produces the gradient instead.  A dropped element of the output is zero, so [H_out > 0] covers
 * the ReLU and the keep mask at once.
 *   COFREE_GRAD_IN_GATED  (GCN, SAGE_CONV): H_in is the output of a layer that ends in ReLU (then dropout);
 *       dH_in is written already multiplied by [H_in > 0] / (1 - dropout_q_below).
 *   COFREE_GRAD_OUT_GATED (act = 1): dH_out arrives already multiplied by [H_out > 0] / (1 - dropout_q) (the
 *       layer above was called with COFREE_GRAD_IN_GATED and this layer's 1/(1-q)); this layer skips its
 *       own pass.
 * Both describe the same gradient with respect to the parameters as the plain calls. */
#define COFREE_GRAD_IN_GATED 1u
#define COFREE_GRAD_OUT_GATED 2u

typedef struct cofree_layer_params { /* device, float32 */
  const float* W;
  const float* bW;
  const float* U;  /* SAGE only */
  const float* bU; /* SAGE only */
} cofree_layer_params;

typedef struct cofree_layer_grads { /* device, float32, same shapes as the parameters */
  float* W;
  float* bW;
  float* U;
  float* bU;
} cofree_layer_grads;

/* Activations kept from forward for backward; device buffers owned by the caller.
 *   SAGE: Z [n_nodes, d_msg] = ReLU(H W^T + bW); A [n_nodes, d_msg] = its neighbourhood mean
 *         (when d_out < d_msg the mean is taken after U_a, which commutes with it, and A is only
 *         used as scratch for Z U_a^T).
 *   GCN : A [n_nodes, d_in] = S(A+I)S.H when d_in <= d_out (aggregate first), unused otherwise; Z unused.
 *   SAGE_CONV: A [n_nodes, d_in] = neighbourhood mean of H when d_in <= d_out, unused otherwise; Z unused. */
typedef struct cofree_layer_saved {
  void* Z;
  void* A;
} cofree_layer_saved;

/* Bytes of scratch a forward (backward = 0) or backward (backward = 1) call needs. */
size_t cofree_layer_workspace_bytes(const cofree_layer_desc* desc, int64_t n_nodes, int32_t backward);

/* H_in [n_nodes, d_in] -> H_out [n_nodes, d_out]; fills `saved`.  workspace: device scratch of
 * at least cofree_layer_workspace_bytes(desc, n_nodes, 0) bytes, 256-byte aligned. */
int32_t cofree_layer_fwd(const cofree_partition* part, const cofree_masks* masks, int32_t mask_id,
                         const cofree_layer_desc* desc, const void* H_in, const cofree_layer_params* params,
                         void* H_out, const cofree_layer_saved* saved, void* workspace, size_t workspace_bytes,
                         void* stream);

/* Backward of the same layer.  dH_out [n_nodes, d_out] is the gradient w.r.t. the layer output;
 * H_in / H_out / saved are the forward call's; dH_in [n_nodes, d_in] receives the gradient
 * w.r.t. the input, or is NULL for the first layer (features need no gradient).  Parameter
 * gradients are written to `grads`, or added to it when accumulate != 0 (gradient sum over
 * partitions, Eq. 2).  Reductions use a fixed order: results are run-to-run identical. */
int32_t cofree_layer_bwd(const cofree_partition* part, const cofree_masks* masks, int32_t mask_id,
                         const cofree_layer_desc* desc, const void* H_in, const void* H_out,
                         const cofree_layer_params* params, const cofree_layer_saved* saved, const void* dH_out,
                         void* dH_in, const cofree_layer_grads* grads, int32_t accumulate, void* workspace,
                         size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------
 * Reweighted loss (Eq. 3):  L = c * sum_{j in V[i]} w_j * CE(softmax(logits_j), labels_j)
 * with w = Degree-Aware Reweighting weights (COFREE_W_DAR), ones (COFREE_W_NONE) or a device
 * vector custom_w [n_nodes] (COFREE_W_CUSTOM).  train_mask (device uint8 [n_nodes], may be NULL)
 * zeroes the weight of unselected nodes.  Writes the float32 loss to the device scalar loss_out
 * and dlogits[j] = c * w_j * (softmax(logits_j) - onehot(labels_j)) (dtype as logits).
 * workspace: device scratch of at least cofree_loss_workspace_bytes() bytes.
 */
size_t cofree_loss_workspace_bytes(void);
int32_t cofree_loss_weighted(const cofree_partition* part, int32_t weight_kind, const float* custom_w,
                             const void* logits, int32_t dtype, const int32_t* labels, const uint8_t* train_mask,
                             int32_t n_classes, float scale_c, float* loss_out, void* dlogits, void* workspace,
                             size_t workspace_bytes, void* stream);

/* cofree_loss_weighted for callers that cannot allocate device memory or hand over a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and kernels
 * as cofree_loss_weighted, minus the workspace: the per-workgroup partial sums (2048 floats, 8 KiB) live in a
 * file-scope device array of the library that every GPU the library runs on holds until the process ends.
 * The call makes no hipMalloc / hipFree and calls no allocating routine; its only set-up is one address
 * look-up per device on the first call there.  Limits: n_classes <= COFREE_LOSS_STATIC_MAX_CLASSES and a
 * partition of at most COFREE_LOSS_STATIC_MAX_NODES nodes, else COFREE_EINVAL; device index below
 * COFREE_STATIC_MAX_DEVICES.  All calls on one GPU share the one array: calls that overlap on a GPU
 * (different streams or host threads) race on it - issue them one after the other on one stream.  Nothing
 * has to be cleared between calls: every partial sum is rewritten before it is read. */
#define COFREE_LOSS_STATIC_MAX_CLASSES 4096
#define COFREE_LOSS_STATIC_MAX_NODES ((int64_t)1 << 27)
#define COFREE_STATIC_MAX_DEVICES 64
int32_t cofree_loss_weighted_static(const cofree_partition* part, int32_t weight_kind, const float* custom_w,
                                    const void* logits, int32_t dtype, const int32_t* labels,
                                    const uint8_t* train_mask, int32_t n_classes, float scale_c, float* loss_out,
                                    void* dlogits, void* stream);

/* Multi-label variant: the sigmoid + binary cross-entropy loss that Theorem 3 is stated for
 * (Section 4.3), summed over the n_classes independent outputs of a node:
 *   L = c * sum_j w_j * sum_k [ softplus(z_jk) - y_jk z_jk ],  dlogits[j,k] = c * w_j * (sigmoid(z_jk) - y_jk).
 * targets: device uint8 [n_nodes, n_classes], non-zero = 1.  Everything else as cofree_loss_weighted. */
int32_t cofree_loss_bce_weighted(const cofree_partition* part, int32_t weight_kind, const float* custom_w,
                                 const void* logits, int32_t dtype, const uint8_t* targets, const uint8_t* train_mask,
                                 int32_t n_classes, float scale_c, float* loss_out, void* dlogits, void* workspace,
                                 size_t workspace_bytes, void* stream);

/* Gradient gap of a cut (the objective of Eq. 2 evaluated for the weights in use):
 * out[0] = || g_full - g_sum ||_F and out[1] = || g_full ||_F over n float32 elements, with g_full the
 * gradient on the uncut graph and g_sum the sum of the partitions' gradients (all device pointers;
 * out: 2 floats).  Fixed-order reduction.  workspace: at least cofree_loss_workspace_bytes() bytes. */
int32_t cofree_grad_gap(int64_t n, const float* g_full, const float* g_sum, float* out, void* workspace,
                        size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------
 * Parameter update over n float32 elements (Algorithm 1 line 11):
 *   COFREE_SGD : theta -= lr * grad                       (m, v unused, may be NULL)
 *   COFREE_ADAM: m = b1 m + (1-b1) g; v = b2 v + (1-b2) g^2;
 *                theta -= lr * (m/(1-b1^t)) / (sqrt(v/(1-b2^t)) + eps),  t >= 1 the step count.
 */
int32_t cofree_step(int32_t kind, int64_t n, float* theta, const float* grad, float* m, float* v, float lr,
                    float b1, float b2, float eps, int64_t t, void* stream);

/* ---------------------------------------------------------------------------------------
 * Dense transform used inside the layers, exposed for direct testing and timing:
 *   C[M,N] = A[M,K] . B^T (+ bias, ReLU),  B [N,K], all float32 device, MFMA with fp32 accumulate.
 */
int32_t cofree_dense_nt_f32(const float* A, const float* B, const float* bias, float* C, int64_t M, int32_t N,
                            int32_t K, int32_t relu, void* stream);

/* ---------------------------------------------------------------------------------------
 * Per-kernel timing for roofline reports (not part of the method).  While enabled, every kernel
 * the library launches is bracketed by HIP events on its stream; cofree_profile_read waits for
 * the recorded events and returns, per kernel name, the launch count, the summed duration and
 * the summed algorithmic bytes / flops of those launches.  cofree_profile_enable clears the
 * records.  Not thread-safe against concurrent launches on other threads' behalf beyond a mutex.
 */
typedef struct cofree_kernel_stat {
  char name[96]; /* kernel template instance and launch shape */
  int64_t launches;
  double ms_total;
  double alg_bytes; /* bytes the launches had to move at minimum (each operand once) */
  double alg_flops; /* floating point operations of the launches */
} cofree_kernel_stat;
int32_t cofree_profile_enable(int32_t on);
int32_t cofree_profile_read(cofree_kernel_stat* out, int32_t max_entries, int32_t* n_out);

#ifdef __cplusplus
}
#endif
#endif /* COFREE_H */
