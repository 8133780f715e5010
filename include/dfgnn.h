/*
 * dfgnn.h - C ABI of the fused attention-GNN graph convolution for AMD MI355X (gfx950).
 *
 * The library computes, for a graph stored as CSR by destination, the three fused steps of an
 * attention-GNN layer (Eq. 1, Sec. 2.1):  S = SDDMM(Q, K, A)  ->  P = Softmax(S) over each node's
 * neighbourhood (Appendix A)  ->  O = SpMM(P, V),  and the backward pass of Appendix B, for the three
 * models of Sec. 5.1: GT (dot-SDDMM), GAT (add-SDDMM) and AGNN (dot-SDDMM on L2-normalised features),
 * and for GATv2 (the other member of the GAT family cited in Sec. 1).
 * Per-edge scores and attention weights live only in registers; nothing of size O(edges) is written
 * to memory by the layer calls (except the gradient of an edge term, when the caller asks for one, and
 * the output of dfgnn_attention_weights, which exists to write them).
 *
 * General rules
 *  - Every pointer named d_* or documented as "device" is GPU global memory owned by the caller; the
 *    library never allocates or frees device memory and keeps only a small host-side handle.
 *  - Node tensors are [N, H, D] row-major (one node's H*D values contiguous), in the layer's dtype
 *    (fp32, bf16 or fp16; the 16-bit types are storage types: all arithmetic and accumulation is fp32 and
 *    results are rounded to nearest even when stored); statistics and attention vectors are fp32.  Device
 *    pointers must be 16-byte aligned.
 *  - Row i of the CSR is destination i; indices[indptr[i] .. indptr[i+1]) are its in-neighbours
 *    (sources).  Sources need not be sorted inside a row; repeated edges are separate softmax terms;
 *    empty rows are legal (O = 0, row_max = -inf, row_sum = 0, no gradient contribution).
 *  - All layer calls are asynchronous on the HIP stream passed as `stream` (a hipStream_t; NULL = the
 *    default stream).  Only dfgnn_graph_create and dfgnn_graph_set_batch synchronise that stream.
 *  - Every function returns a dfgnn_status; nothing throws or aborts across this boundary.  On any
 *    error no output buffer has defined contents.  dfgnn_last_error() gives a thread-local detail text.
 *  - Outputs are overwritten, never accumulated into.
 *  - A graph with N = 0 is legal: layer calls then touch no node tensor (their pointers may be NULL).
 */
#ifndef DFGNN_H
#define DFGNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DFGNN_OK = 0,
    DFGNN_EINVAL = 1,       /* NULL pointer, negative size, inconsistent arguments, malformed graph */
    DFGNN_EUNSUPPORTED = 2, /* shape / dtype / alignment the kernels do not cover                    */
    DFGNN_EWORKSPACE = 3,   /* a caller-provided buffer is too small                                 */
    DFGNN_EHIP = 4          /* a HIP runtime call failed (text in dfgnn_last_error)                  */
} dfgnn_status;

typedef enum { DFGNN_GT = 0, DFGNN_GAT = 1, DFGNN_AGNN = 2, DFGNN_GATV2 = 3 } dfgnn_model;
typedef enum { DFGNN_F32 = 0, DFGNN_BF16 = 1, DFGNN_F16 = 2 } dfgnn_dtype;

/*
 * Degree-aware scheduling parameters.  The switch between one fused node-parallel pass and an
 * edge-parallel treatment of super nodes (Sec. 3, Sec. 4.2 "SDDMM") is taken per row here: a row with
 * at least super_threshold neighbours is cut into chunks of chunk_edges edges whose partial softmax
 * statistics are merged in a second pass.  0 selects the library default for either field:
 * chunk_edges = E / 16384 rounded up to a power of two and clamped to [128, 512] (E = edges of the
 * graph), super_threshold = 2 * chunk_edges.  The values in use can be read with dfgnn_graph_query.
 */
typedef struct {
    int32_t super_threshold;
    int32_t chunk_edges;
    int32_t flags;       /* DFGNN_SCHED_* bits; 0 = default behaviour */
    int32_t reserved[5]; /* must be 0 */
} dfgnn_sched_params;

/* Ablation switch: rows shorter than one load round of a wavefront are normally mapped one per
 * edge slot (several rows per wavefront); with this bit every row below super_threshold gets a whole
 * wavefront.  Results are the same up to rounding order. */
#define DFGNN_SCHED_NO_SHORT_ROWS 1
/* Ablation switch: do not use the dense-tile kernels for batches of small graphs (dfgnn_graph_set_batch). */
#define DFGNN_SCHED_NO_DENSE_BATCH 2
/* Use the dense-tile kernels whenever they apply, also below the tile fill from which they pay. */
#define DFGNN_SCHED_FORCE_DENSE_BATCH 4
/* Comparator for the fusion study (Sec. 3, "parallelism maximization fusion"; ablation of Appendix C):
 * the GT forward pass runs as two kernels, an edge-parallel SDDMM over a COO row array that writes the
 * E x H fp32 scores to the workspace, and a softmax + SpMM kernel that reads them back.  Costs one more
 * int32 per edge of graph metadata and E*H*4 bytes of forward workspace; results are the same up to
 * rounding order.  Other models, the backward pass and the dense-tile kernels are unaffected. */
#define DFGNN_SCHED_SCORES_IN_MEMORY 8
/* Ablation switch.  dfgnn_graph_create samples the edges; when at least half of them connect nodes whose
 * ids differ by less than 4096 (batches of small graphs, meshes, clustered numberings) the layer launches
 * keep runs of 32 consecutive workgroups of their work list on one XCD, so that rows which share
 * neighbours share an L2.  With this bit workgroups are dealt round-robin for every graph.  Results are
 * bit-identical either way. */
#define DFGNN_SCHED_NO_XCD_GROUPS 16
/* Forward-only graph (inference): dfgnn_graph_create builds neither the CSC transpose nor the column
 * schedule, which are most of its work and the two edge-sized arrays of its metadata
 * (dfgnn_graph_meta_bytes shrinks accordingly).  dfgnn_forward*, dfgnn_attention_weights and
 * dfgnn_graph_set_batch work as usual; dfgnn_backward* return EINVAL; the CSC items of dfgnn_graph_query
 * have count 0. */
#define DFGNN_SCHED_FORWARD_ONLY 32
/* Ablation switch.  For small fp32 GT graphs (at most 262144 edges, no super rows or columns, no edge term) the
 * backward call runs its row side and its column side as one launch: the column side recomputes the softmax
 * statistics and delta_i = dO_i . O_i of every edge's row from the forward results instead of waiting for the
 * row side to hand them over.  With this bit the two sides are separate launches for every graph.  Results
 * are the same up to rounding order. */
#define DFGNN_SCHED_NO_PAIRED_PASSES 64

/* One layer call's model description. */
typedef struct {
    int32_t model;   /* dfgnn_model */
    int32_t dtype;   /* dfgnn_dtype of node tensors (inputs, outputs and their gradients) */
    int32_t H;       /* heads */
    int32_t D;       /* features per head; D * sizeof(element) must be a multiple of 16 bytes, D/vec a power
                        of two (vec = 4 for fp32, 8 for bf16 and fp16) and at most 64 (one head fits one wavefront of
                        16-byte lanes: D <= 256 in fp32, 512 in bf16 / fp16).  Node tensors (N*H*D elements) of
                        4 GiB and more are taken by a slower set of kernels (64-bit gather addresses, head
                        reductions by shuffles) as long as N*H*16 bytes stay below 4 GiB; the dense-tile batch
                        kernels are unaffected.  Rows of more than 64 such lanes (H*D/vec > 64) are processed
                        in groups of heads, one launch sequence per group.  Other head widths (a classifier
                        layer with 7 outputs, say) are used zero-padded to the next accepted width: zero
                        features change no score of any model and aggregate to zero. */
    float scale;     /* GT: factor on q.k (callers pass 1/sqrt(D)); AGNN: beta; GAT, GATv2: ignored */
    float neg_slope; /* GAT, GATv2: LeakyReLU slope (derivative at 0 is neg_slope) */
    float eps;       /* AGNN: lower clamp of the feature norm */
    int32_t reserved[1];
} dfgnn_layer;

typedef struct dfgnn_graph dfgnn_graph; /* opaque host handle over caller-owned device metadata */

/* Items of dfgnn_graph_query.  Arrays are int32 in device memory inside the metadata buffer. */
typedef enum {
    DFGNN_Q_ROW_ORDER = 0,     /* [N]   rows: super rows (ascending id) first, then by descending bit_length(degree), stable */
    DFGNN_Q_ROW_CHUNK_PTR = 1, /* [n_super_rows + 1] first chunk of every super row */
    DFGNN_Q_ROW_CHUNKS = 2,    /* [n_row_chunks * 3] (row, begin, end) CSR edge ranges */
    DFGNN_Q_T_INDPTR = 3,      /* [N + 1] CSC pointer (by source) */
    DFGNN_Q_T_INDICES = 4,     /* [E]   destination of every out-edge, columns ascending, CSR position ascending inside a column */
    DFGNN_Q_T_EID = 5,         /* [E]   CSR position of every CSC entry */
    DFGNN_Q_COL_ORDER = 6,     /* [N]   same ordering rule applied to out-degrees */
    DFGNN_Q_COL_CHUNK_PTR = 7, /* [n_super_cols + 1] */
    DFGNN_Q_COL_CHUNKS = 8,    /* [n_col_chunks * 3] (column, begin, end) CSC entry ranges */
    DFGNN_Q_N_SUPER_ROWS = 9,  /* count only (d_ptr = NULL) */
    DFGNN_Q_N_SUPER_COLS = 10, /* count only */
    DFGNN_Q_SUPER_THRESHOLD = 11, /* count only: the super_threshold in use */
    DFGNN_Q_CHUNK_EDGES = 12,     /* count only: the chunk_edges in use */
    DFGNN_Q_BATCH_DENSE = 13,     /* count only: 1 if the dense-tile batch kernels apply to this graph */
    DFGNN_Q_XCD_GROUP = 14        /* count only: workgroups per XCD-local run (0: the numbering is not local) */
} dfgnn_query;

const char* dfgnn_status_string(int status);
const char* dfgnn_last_error(void); /* never NULL; valid until the calling thread's next library call */
int dfgnn_version(int* major, int* minor);
/* Hash of the source files, this header and the compiler flags the library was built from (set by the build
 * script; "unknown" for other builds).  Lets a test harness refuse a library that is older than the sources. */
const char* dfgnn_build_id(void);

/*
 * Scheduler metadata (the preprocessing step of Sec. 5.3: CSR for the forward pass, CSC for the
 * backward pass, plus the per-row work classification that replaces the whole-graph strategy switch
 * of Sec. 4.2).
 *
 * dfgnn_graph_meta_bytes: sizes of the two device buffers dfgnn_graph_create needs for a graph of N
 *   nodes and E edges: meta_bytes (lives as long as the graph handle) and scratch_bytes (used only
 *   during creation).  sched may be NULL (defaults).  Host-only; needs no GPU.
 *
 * dfgnn_graph_create: validates the CSR (monotone indptr starting at 0 and ending at E, indices in
 *   [0, N)), then builds on the GPU: the row order, the super-row chunk list, the CSC transpose
 *   (out-edges of a source listed in increasing CSR position) and the same order / chunk list for
 *   columns.  d_indptr [N+1] and d_indices [E] are device int32, caller-owned, and must stay valid and
 *   unchanged while the handle is used.  Requires 0 <= N, 0 <= E < 2^31 - 2^20.  Synchronises `stream`.
 *   Errors: EINVAL (NULL / negative / malformed CSR), EWORKSPACE (buffers smaller than
 *   dfgnn_graph_meta_bytes reports), EHIP.  On success *out receives a handle to be released with
 *   dfgnn_graph_destroy (host memory only; device buffers stay the caller's).
 *
 * dfgnn_graph_query: device pointer and element count of one metadata array (for bit-exact checks).
 */
int dfgnn_graph_meta_bytes(int64_t N, int64_t E, const dfgnn_sched_params* sched, size_t* meta_bytes,
                           size_t* scratch_bytes);
int dfgnn_graph_create(dfgnn_graph** out, int64_t N, int64_t E, const int32_t* d_indptr, const int32_t* d_indices,
                       const dfgnn_sched_params* sched, void* d_meta, size_t meta_bytes, void* d_scratch,
                       size_t scratch_bytes, void* stream);
int dfgnn_graph_destroy(dfgnn_graph* graph);

/*
 * Batched small graphs (the batch-graph workloads of Sec. 5.1: many small graphs processed as one
 * block-diagonal graph).  d_batch_ptr [n_graphs + 1] (device int32, caller-owned) holds the first node of
 * every graph: graph b owns nodes [batch_ptr[b], batch_ptr[b+1]).  d_batch is a device buffer of at
 * least dfgnn_graph_batch_bytes(N, n_graphs) bytes, 256-byte aligned; it and d_batch_ptr must stay valid
 * while the handle is used.  The call checks on the GPU that the pointer array starts at 0, ends at N and
 * does not decrease and that no edge connects two graphs (EINVAL otherwise), and records for each row
 * and each column its adjacency bits inside its graph.
 * If no edge is repeated, GT layers are then computed by dense-tile kernels when that pays, i.e. when the
 * 16 x 16 score tiles of the graphs are full enough (edges / (256 x number of tiles) at least about 0.2; below that the general kernels are faster):
 *   bf16, D = 16 or 32, graphs of at most 64 nodes: one wavefront per (graph, head) stages the head's
 *     Q, K, V once into LDS and forms the masked score block with MFMA;
 *   fp32 or bf16, D = 16, 32 or 64, graphs of at most 512 nodes: one wavefront per (graph, head, 16
 *     rows) streams over the graph's column tiles with MFMA.
 * Every node row is then read once per graph (or once per row tile) instead of once per edge; results
 * agree with the general path to rounding.  Other layers, and batches that do not qualify, use the
 * general kernels unchanged.  Passing (NULL, 0, NULL, 0) forgets the batch structure.  Synchronises
 * `stream`.  Errors: EINVAL, EWORKSPACE, EHIP.
 */
int dfgnn_graph_batch_bytes(int64_t N, int64_t n_graphs, size_t* batch_bytes);
int dfgnn_graph_set_batch(dfgnn_graph* graph, const int32_t* d_batch_ptr, int64_t n_graphs, void* d_batch,
                          size_t batch_bytes, void* stream);
int dfgnn_graph_query(const dfgnn_graph* graph, int what, const void** d_ptr, int64_t* count);

/*
 * dfgnn_graph_create and dfgnn_graph_set_batch in one call, for the batch-graph setting of Sec. 5.1, where
 * the preprocessing of Sec. 5.3 (CSR, CSC, schedule) is paid for every mini-batch and has to cost about
 * what a training step costs.  Arguments as in those two calls; the result (every metadata array, the
 * batch tables) is bit for bit what they would produce.  When every graph of the batch has at most 4096
 * nodes and 65536 edges the metadata is built by one workgroup per graph in three launches with one
 * synchronisation of `stream` (two when the batch has super rows or columns); other batches, forward-only
 * graphs and the scores-in-memory comparator go through the two general calls internally.
 * dfgnn_graph_create itself builds a graph of at most 4096 nodes and 65536 edges (without batch
 * structure) the same way, in one launch.
 * Errors: those of dfgnn_graph_create and dfgnn_graph_set_batch.
 */
int dfgnn_graph_create_batch(dfgnn_graph** out, int64_t N, int64_t E, const int32_t* d_indptr, const int32_t* d_indices,
                             const int32_t* d_batch_ptr, int64_t n_graphs, const dfgnn_sched_params* sched, void* d_meta,
                             size_t meta_bytes, void* d_batch, size_t batch_bytes, void* d_scratch, size_t scratch_bytes,
                             void* stream);

/*
 * Bytes of device workspace one forward / one backward call needs for this graph and layer (partial
 * results of super-row chunks, statistics and per-node terms handed from the row pass to the column
 * pass, reduction staging).  Either output pointer may be NULL.  Errors: EINVAL, EUNSUPPORTED.
 */
int dfgnn_workspace_bytes(const dfgnn_graph* graph, const dfgnn_layer* layer, size_t* fwd_bytes, size_t* bwd_bytes);

/*
 * Forward: O_i = sum_{j in N(i)} softmax_j(s_ij) Val_j per head (Eq. 1; edge softmax of Appendix A).
 *   GT   s_ij = scale * q_i . k_j                         x = Q, k = K, v = V (Val = V)
 *   GAT  s_ij = LeakyReLU(a_l . Wh_i + a_r . Wh_j)        x = Wh, a_l, a_r [H, D] fp32 device (Val = Wh); k = v = NULL
 *   AGNN s_ij = beta * cos(h_i, h_j) per head             x = h (Val = h, un-normalised); k = v = a_r = NULL; a_l = NULL (beta is
 *                                                         layer->scale) or a device pointer to one fp32 value that holds beta
 *                                                         (layer->scale is ignored then: a trained beta stays on the device and
 *                                                         the call can be recorded into a HIP graph); the same in dfgnn_backward
 *                                                         and dfgnn_attention_weights
 *   GATv2 s_ij = sum_d a_d LeakyReLU(x_i,d + k_j,d)       x = destination-side, k = source-side projection of the
 *        (the other member of the GAT family cited in       node features (Val = k), a_l = a [H, D] fp32 device;
 *         Sec. 1; its score is not separable per node)       v = a_r = NULL
 * out [N,H,D] in the layer dtype; row_max, row_sum [N,H] fp32 are the softmax statistics
 * (max_j s_ij and sum_j exp(s_ij - max)) that dfgnn_backward consumes.
 * workspace: device, >= fwd_bytes of dfgnn_workspace_bytes, 256-byte aligned, contents undefined on
 * entry and exit.  Errors: EINVAL, EUNSUPPORTED, EWORKSPACE, EHIP.
 */
int dfgnn_forward(const dfgnn_graph* graph, const dfgnn_layer* layer, const void* x, const void* k, const void* v,
                  const float* a_l, const float* a_r, void* out, float* row_max, float* row_sum, void* workspace,
                  size_t workspace_bytes, void* stream);

/*
 * dfgnn_forward for callers that cannot allocate device memory for a workspace (code recorded under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): the same computation with the same
 * kernels and bit-identical results, but the chunk partials of super rows are kept in a static device
 * array of DFGNN_STATIC_SCRATCH_BYTES owned by the library (each GPU that uses the library holds it until
 * the process ends).  The call allocates and frees nothing, on the host side of HIP or on the device.
 *  - Limit: the forward workspace of this graph and layer (fwd_bytes of dfgnn_workspace_bytes) must not
 *    exceed DFGNN_STATIC_SCRATCH_BYTES, else EWORKSPACE and nothing is launched (about 29,000 chunks of
 *    128-feature rows; graphs with more chunk work need dfgnn_forward and a caller workspace).
 *  - The GPU of `stream` must be the calling thread's current device.  The first call on a GPU looks up the
 *    array's address there; make that first call outside stream capture.
 *  - Every call on one GPU shares that GPU's array: calls that may overlap on one GPU (different streams,
 *    different threads) race and must be ordered by the caller.  Calls on one stream are ordered already.
 *  - The array keeps the previous call's contents; the forward pass needs no part of it cleared.
 * Arguments, layouts and errors otherwise as dfgnn_forward.
 */
#define DFGNN_STATIC_SCRATCH_BYTES (16u << 20)
int dfgnn_forward_static(const dfgnn_graph* graph, const dfgnn_layer* layer, const void* x, const void* k,
                         const void* v, const float* a_l, const float* a_r, void* out, float* row_max,
                         float* row_sum, void* stream);

/*
 * Backward (Appendix B; the fused SDDMM -> softmax-backward -> SpMM chain of Sec. 4.3 over the CSR,
 * and the transposed products over the CSC).  Inputs are those of the forward call plus its results
 * out, row_max, row_sum and the upstream gradient d_out = dL/dO [N,H,D].
 *   GT   -> d_x = dL/dQ, d_k = dL/dK, d_v = dL/dV                        (d_a_l = d_a_r = d_scale = NULL)
 *   GAT  -> d_x = dL/dWh, d_a_l, d_a_r [H,D] fp32                        (d_k = d_v = d_scale = NULL)
 *   AGNN -> d_x = dL/dh, d_scale = dL/dbeta (1 float, device)            (d_k = d_v = d_a_l = d_a_r = NULL; a_l as in dfgnn_forward)
 *   GATv2 -> d_x, d_k (destination- and source-side), d_a_l = dL/da      (d_v = d_a_r = d_scale = NULL)
 * Gradient node tensors are in the layer dtype.  workspace: >= bwd_bytes, 256-byte aligned.
 * Results are deterministic (no floating-point atomics).
 */
int dfgnn_backward(const dfgnn_graph* graph, const dfgnn_layer* layer, const void* x, const void* k, const void* v,
                   const float* a_l, const float* a_r, const void* out, const float* row_max, const float* row_sum,
                   const void* d_out, void* d_x, void* d_k, void* d_v, float* d_a_l, float* d_a_r, float* d_scale,
                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same two calls with an additive per-edge term in the score (edge features entering the attention
 * score, Sec. 1): s_ij = (model score) + edge_bias[t, h] for the edge stored at CSR position t, before the
 * edge softmax of Appendix A.  edge_bias: [E, H] fp32 device, caller-owned, in the order of d_indices;
 * NULL = no edge term (then the calls are dfgnn_forward / dfgnn_backward); E*H*4 bytes must stay below
 * 4 GiB.  d_edge_bias: [E, H] fp32 device, receives dL/d edge_bias = dS of every edge (Appendix B's dL/dS
 * before it is multiplied into Q and K); may be NULL when the term is not trained.  Works for every
 * model; batches of small graphs use the general kernels when an edge term is given (the dense-tile
 * kernels have none).  Same errors as above.
 */
int dfgnn_forward_edge_bias(const dfgnn_graph* graph, const dfgnn_layer* layer, const void* x, const void* k,
                            const void* v, const float* a_l, const float* a_r, const float* edge_bias, void* out,
                            float* row_max, float* row_sum, void* workspace, size_t workspace_bytes, void* stream);
int dfgnn_backward_edge_bias(const dfgnn_graph* graph, const dfgnn_layer* layer, const void* x, const void* k,
                             const void* v, const float* a_l, const float* a_r, const float* edge_bias,
                             const void* out, const float* row_max, const float* row_sum, const void* d_out, void* d_x,
                             void* d_k, void* d_v, float* d_a_l, float* d_a_r, float* d_scale, float* d_edge_bias,
                             void* workspace, size_t workspace_bytes, void* stream);

/*
 * Attention weights (the normalised scores P = Softmax(S) of Eq. 1, which the fused layer never writes):
 * p[t, h] = exp(s_ij - row_max[i, h]) / row_sum[i, h] for the edge i <- j stored at CSR position t, from
 * the inputs and the statistics of a finished dfgnn_forward (or dfgnn_forward_edge_bias; pass the same
 * edge_bias, or NULL) call.  p: [E, H] fp32 device, caller-owned, every entry is overwritten.  Tensor
 * arguments as in dfgnn_forward for the model (v is not needed).  Needs no workspace.  One gather pass
 * over the CSR; meant for inspection (attention maps): the layer's own backward pass never needs it and
 * the library has no gradient through this output.  Errors: EINVAL, EUNSUPPORTED, EHIP.
 */
int dfgnn_attention_weights(const dfgnn_graph* graph, const dfgnn_layer* layer, const void* x, const void* k,
                            const float* a_l, const float* a_r, const float* edge_bias, const float* row_max,
                            const float* row_sum, float* p, void* stream);

/*
 * Optional per-kernel timing for benchmarks (the measurement protocol of Sec. 5.2 reports kernel time).
 * dfgnn_timing_enable(1) makes every later layer call record a pair of HIP events around each kernel
 * it launches, on the stream of that call; dfgnn_timing_enable(0) stops it.  Either call discards
 * what was recorded.  Process-wide switch, not thread-safe; off by default (no events, no overhead).
 * dfgnn_timing_collect waits for the recorded events, sums the elapsed milliseconds per kernel label
 * into the caller's host arrays (at most max_labels entries; labels are static strings owned by the
 * library), stores the number of labels in *n_labels and clears the record list.  At most 65536
 * launches are recorded between two collects; later ones are not timed.
 * Errors: EINVAL (NULL), EWORKSPACE (more labels than max_labels), EHIP.
 */
int dfgnn_timing_enable(int enable);
int dfgnn_timing_collect(int max_labels, const char** labels, double* total_ms, int64_t* launches, int* n_labels);

/*
 * Measurement yardstick, not part of the layer (Sec. 5.2 reports bandwidth utilisation; this gives the rate
 * the memory system sustains for the access pattern the layer is made of).  Reads row idx[e] of `table`
 * (device, n_rows rows of row_bytes bytes, row_bytes = 16, 32, ..., 1024; below 4 GiB in all) for every
 * e < n_idx with the gather instruction of the pass kernels, one row per group of row_bytes / 16 lanes, and
 * does nothing else with it; an index outside [0, n_rows) reads nothing.  `idx`: device, int32[n_idx].
 * `out`: device scratch of the caller, out_bytes >= 4096; every 4096 bytes of it make one workgroup of 4
 * wavefronts, each thread leaves the XOR of the 16-byte pieces it read there (16 bytes per thread), so the
 * caller chooses the size of the launch.  Asynchronous on `stream`.  Errors: EINVAL, EUNSUPPORTED, EHIP.
 */
int dfgnn_probe_gather(const void* table, int64_t n_rows, int32_t row_bytes, const int32_t* idx, int64_t n_idx,
                       void* out, size_t out_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DFGNN_H */
