/*
 * dgi.h — C ABI of the layer-wise full-graph GNN inference library for MI355X (gfx950).
 *
 * The library runs the layer-wise schedule of the DGI paper (arXiv 2211.15082, Section 2,
 * Algorithm 2): every layer is evaluated once over all nodes, in batches of destination
 * nodes; a batch gathers only the 1-hop in-neighbours of its nodes (Eq. 1), so the L-hop
 * neighbour explosion of node-wise inference (Algorithm 1) never arises.  Graph, features,
 * weights and every intermediate embedding are resident in HBM; the "copy to the computing
 * device" steps of Algorithm 2 therefore vanish and a batch is a range of CSR rows.
 *
 * Conventions
 *   - All pointers are plain pointers.  Each argument says HOST or DEVICE.  DEVICE pointers
 *     are HIP device allocations of the current device (e.g. a torch tensor's data_ptr()).
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls that
 *     take a stream enqueue work on it and return without waiting unless stated otherwise.
 *   - Matrices are row-major with an explicit leading dimension `ld` counted in ELEMENTS.
 *   - Every call returns a dgi_status_t; nothing throws or aborts across this boundary.  The
 *     text of the last failure on the calling thread is available from dgi_last_error().
 *   - The library never takes ownership of caller memory.  Handles it returns are released
 *     with the matching *_free call.
 */
#ifndef DGI_H
#define DGI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DGI_VERSION_MAJOR 0
#define DGI_VERSION_MINOR 1
#define DGI_MAX_LAYERS 16

typedef enum {
    DGI_OK = 0,
    DGI_ERR_INVALID_ARG = 1, /* NULL where data is required, negative size, bad range, dims that disagree */
    DGI_ERR_BAD_GRAPH = 2,   /* indptr not monotone / indptr[0]!=0 / indptr[N]!=E / index out of [0,N) */
    DGI_ERR_UNSUPPORTED = 3, /* dtype / aggregator / order combination the kernels do not implement */
    DGI_ERR_OOM = 4,         /* workspace does not fit the budget even at one row per batch (Sec. 4.1) */
    DGI_ERR_DEVICE = 5       /* a HIP call failed; dgi_last_error() holds its text */
} dgi_status_t;

typedef enum { DGI_I32 = 0, DGI_I64 = 1 } dgi_itype_t;
typedef enum { DGI_HOST = 0, DGI_DEVICE = 1 } dgi_memloc_t;
typedef enum { DGI_F32 = 0, DGI_BF16 = 1 } dgi_dtype_t;

/* AGGREGATE of Eq. 1.  N(v) = in-neighbours of v = the entries of CSR row v.
 *   SUM : m_v = sum_u h_u                      MEAN: m_v = (1/|N(v)|) sum_u h_u   (0 if N(v) empty)
 *   GCN : m_v = sum_u h_u / sqrt(d_out(u) d_in(v)), degrees counted on the stored CSR, clamped >= 1
 *   GAT : m_v = concat_h sum_u alpha^h_uv z^h_u, alpha = softmax_u LeakyReLU(<a_src^h,z^h_u> + <a_dst^h,z^h_v>)
 * SUM/MEAN: h'_v = act(h_v W_self + m_v W_neigh + b)  (W_self may be NULL: term dropped)
 * GCN     : h'_v = act(m_v W_neigh + b)
 * GAT     : z = h W_neigh viewed as [heads, head_dim];  h'_v = act(m_v + b)                              */
typedef enum { DGI_AGG_SUM = 0, DGI_AGG_MEAN = 1, DGI_AGG_GCN = 2, DGI_AGG_GAT = 3 } dgi_agg_t;

typedef enum { DGI_ACT_NONE = 0, DGI_ACT_RELU = 1, DGI_ACT_ELU = 2, DGI_ACT_LEAKY_RELU = 3 } dgi_act_t;

/* Whether the dense transform runs before or after the neighbour aggregation.  Both give the same
 * result up to rounding, because aggregation is linear.  AUTO = transform first iff out_dim < in_dim
 * (GAT is always transform-first).  An aggregate-first layer runs either as one kernel that keeps the
 * aggregated tile in LDS and feeds it to the matrix cores (FUSED), or as an aggregation kernel followed by a
 * GEMM (SPLIT); AUTO and AGG_FIRST choose between the two from the graph's average degree and the layer
 * widths.  FUSED falls back to SPLIT for layouts the fused kernel does not take (rows not 16-byte aligned,
 * in_dim not a multiple of 16 bytes or at most 8 x 16 bytes, tile larger than LDS). */
typedef enum {
    DGI_ORDER_AUTO = 0, DGI_ORDER_AGG_FIRST = 1, DGI_ORDER_TRANSFORM_FIRST = 2,
    DGI_ORDER_AGG_FIRST_FUSED = 3, DGI_ORDER_AGG_FIRST_SPLIT = 4
} dgi_order_t;

/* Node renumbering used to form batches of consecutive ids that share in-neighbours (Section 4.2).
 *   DEGREE : descending in-degree, ties by old id ("Degree Sorting" of Section 5.3)
 *   BFS_RCM: reverse Cuthill-McKee style BFS enumeration on the undirected structure (the paper's RCMK)
 *   RANDOM : seeded shuffle (the "Random" comparison point)
 *   COMMUNITY: ids grouped by the label that DGI_COMMUNITY_ROUNDS rounds of label propagation on the undirected
 *            structure leave on every node (each node repeatedly takes the most frequent label among its in- and
 *            out-neighbours), ties inside a group by old id.  A BFS frontier mixes the communities of a graph after a
 *            few levels; this keeps each one contiguous, which is what makes a batch of consecutive ids share its
 *            in-neighbours when the graph has communities.  Not one of the paper's orderings (Section 4.2 compares
 *            RCMK with Random, Degree Sorting and Rabbit Order): a cheap stand-in for the community-based class. */
typedef enum { DGI_REORDER_NONE = 0, DGI_REORDER_DEGREE = 1, DGI_REORDER_BFS_RCM = 2, DGI_REORDER_RANDOM = 3,
               DGI_REORDER_COMMUNITY = 4 } dgi_reorder_t;
#define DGI_COMMUNITY_ROUNDS 10

typedef struct dgi_graph dgi_graph_t; /* opaque; owns device copies of the CSR and degree vectors */

/* One GNN layer (Eq. 1 instantiated).  All weight pointers are DEVICE pointers, row-major
 * [in_dim x out_dim], so that a row vector h maps to h W.  Weights have dtype `feat_dtype`
 * (fp32, or bf16 stored as uint16 bit patterns); bias and attention vectors are always fp32. */
typedef struct {
    int32_t agg;         /* dgi_agg_t */
    int32_t act;         /* dgi_act_t, applied last */
    float   act_slope;   /* LEAKY_RELU negative slope; ELU alpha */
    int32_t in_dim;
    int32_t out_dim;     /* GAT: heads * head_dim */
    int32_t heads;       /* GAT only; otherwise ignored (use 1) */
    int32_t feat_dtype;  /* dgi_dtype_t of h_in and of the weights */
    int32_t out_dtype;   /* dgi_dtype_t of h_out */
    int32_t order;       /* dgi_order_t */
    const void*  W_self;   /* [in_dim x out_dim] or NULL.  SUM/MEAN only. */
    const void*  W_neigh;  /* [in_dim x out_dim]; the only weight of GCN and GAT */
    const float* bias;     /* [out_dim] or NULL */
    const float* attn_src; /* [heads x head_dim], GAT only */
    const float* attn_dst; /* [heads x head_dim], GAT only */
    float   attn_slope;    /* LeakyReLU slope of the GAT edge score (0.2 in the usual model) */
    int32_t reserved;
} dgi_layer_t;

/* Per-layer measurements filled by dgi_infer when opts->stats is set.  Kernel times are taken with
 * HIP events recorded on the caller's stream around every launch of that kernel class. */
typedef struct {
    int32_t num_layers;
    int32_t reserved;
    double  total_ms;                       /* whole dgi_infer, first enqueue to last completion */
    double  layer_ms[DGI_MAX_LAYERS];
    double  agg_ms[DGI_MAX_LAYERS];         /* the layer's main gather kernel (aggregate, fused aggregate+transform, or
                                               GAT edge kernel), summed over batches; one launch per batch */
    double  hub_ms[DGI_MAX_LAYERS];         /* fused layers only: the hub pre-pass (chunk launch + reduce), summed over batches */
    double  gemm_ms[DGI_MAX_LAYERS];        /* dense transform kernels, summed over batches */
    int64_t agg_launches[DGI_MAX_LAYERS];
    int64_t gemm_launches[DGI_MAX_LAYERS];
    int64_t batches[DGI_MAX_LAYERS];
    int64_t edges[DGI_MAX_LAYERS];          /* edges aggregated by the layer (= E for full inference) */
    int32_t transform_first[DGI_MAX_LAYERS];
    int32_t gather_width[DGI_MAX_LAYERS];   /* elements per gathered source row */
    int32_t fused[DGI_MAX_LAYERS];          /* 1: aggregation and transform ran as one kernel (its time is in agg_ms) */
    int64_t oom_retries;                    /* batches redone after halving the thresholds (Sec. 4.1) */
    int64_t workspace_bytes;                /* peak bytes the library allocated for this call */
} dgi_stats_t;

typedef struct {
    int64_t batch_size;            /* destination rows per batch; 0 = dynamic control of Sec. 4.1 (Eq. 2) */
    const int32_t* perm_new_of_old;/* DEVICE, N entries, or NULL.  When set, `g` must be the reordered graph
                                      returned by dgi_graph_reorder; x and out stay in ORIGINAL node order and
                                      the library permutes rows on the way in and back on the way out. */
    uint64_t mem_budget_bytes;     /* bytes the call may allocate for hidden layers + temporaries;
                                      0 = 90 % of the currently free device memory (Sec. 4.1) */
    dgi_stats_t* stats;            /* HOST, or NULL.  Setting it makes dgi_infer wait for completion. */
    int64_t init_node_threshold;   /* initial n_t of Eq. 2 for batch_size==0; 0 = 65536.  dgi_infer knows a planned batch's
                                      temporaries before it runs, so the first batch of a layer is rescaled by Eq. 2 on its
                                      plan (it is not launched undersized); dgi_infer_host rescales after each batch */
    int64_t init_edge_threshold;   /* initial n_i of Eq. 2; 0 = init_node_threshold * average degree */
    int32_t jk_concat;             /* 1: jumping-knowledge stack (the paper's JKNet): layers 0..L-2 form a chain and the
                                      last layer reads the concatenation of all their outputs, so layers[L-1].in_dim must
                                      be the sum of the earlier out_dims; every hidden layer is kept until the last
                                      layer has run */
    int32_t host_stream_always;    /* dgi_infer_host only.  1: keep the hidden layers in host memory and stream every
                                      batch (the paper's regime) even when everything would fit the budget */
} dgi_infer_opts_t;

typedef struct {
    int64_t num_nodes;
    int64_t num_edges;
    int64_t max_in_degree;
    int64_t num_hub_rows;     /* rows long enough to be split over several workgroups */
    int64_t num_hub_edges;    /* in-edges of those rows */
    int32_t indptr_type;      /* dgi_itype_t */
    int32_t reserved;
    uint64_t device_bytes;    /* device memory owned by the handle */
} dgi_graph_info_t;

/* ------------------------------------------------------------------------------------------------
 * Graph (the input "G" of Section 2).  CSR keyed by DESTINATION: row v = indices[indptr[v] ..
 * indptr[v+1]) lists the sources u of the edges u->v, i.e. the in-neighbours N(v) of Eq. 1.
 * Duplicate entries are legal and count with multiplicity; rows need not be sorted.
 *   indptr : N+1 entries of type `indptr_type`;  indices: E int32 entries;  both at `where`.
 *   HOST input is copied to the device.  DEVICE input is BORROWED: the caller keeps it alive and
 *   unchanged until dgi_graph_free.  The call validates the CSR (DGI_ERR_BAD_GRAPH otherwise),
 *   computes in/out degrees and their inverse square roots, and finds the hub rows.  It waits
 *   for its own work on `hip_stream` before returning.  N == 0 is legal.                         */
dgi_status_t dgi_graph_load(int64_t num_nodes, int64_t num_edges, const void* indptr, int32_t indptr_type,
                            const int32_t* indices, int32_t where, void* hip_stream, dgi_graph_t** out);
dgi_status_t dgi_graph_free(dgi_graph_t* g);            /* NULL is a no-op; also frees the cached workspace */
/* Frees the buffers dgi_infer and dgi_infer_host keep in the handle between calls (waits for the device first). */
dgi_status_t dgi_graph_release_workspace(dgi_graph_t* g);
dgi_status_t dgi_graph_info(const dgi_graph_t* g, dgi_graph_info_t* info /*HOST*/);

/* Copies of the handle's device vectors for inspection/tests: kind 0 = in-degree (int32), 1 = out-degree
 * (int32), 2 = in-degree^-1/2 (fp32), 3 = out-degree^-1/2 (fp32); `dst` is a HOST buffer of N entries. */
dgi_status_t dgi_graph_vector(const dgi_graph_t* g, int32_t kind, void* dst);
/* Copy the handle's CSR back to HOST buffers (indptr as int64, N+1 entries; indices E entries). */
dgi_status_t dgi_graph_csr(const dgi_graph_t* g, int64_t* indptr, int32_t* indices);

/* Node reordering (Section 4.2).  Builds a renumbered copy of `g` (rows permuted, sources relabelled,
 * each row sorted by new source id) and writes perm_new_of_old[old] = new into a buffer of N int32 at
 * `perm_where` (HOST or DEVICE).  Any bijection leaves the inference result unchanged up to rounding;
 * only locality differs.  DEGREE, BFS_RCM and COMMUNITY permutations are computed on the device (on the
 * host, by the same rule, for graphs beyond the device routines' 2^30-edge limit); relabelling runs on the device.
 * `seed` is used by RANDOM only. */
dgi_status_t dgi_graph_reorder(const dgi_graph_t* g, int32_t method, uint64_t seed, void* hip_stream,
                               dgi_graph_t** g_out, int32_t* perm_new_of_old, int32_t perm_where);

/* ------------------------------------------------------------------------------------------------
 * One layer of Eq. 1 for the destination rows [dst_begin, dst_end) (lines 4-10 of Algorithm 2 for
 * one batch).  h_in  : DEVICE, all N rows of H^{l-1}, [N x in_dim], leading dimension ld_in.
 *              h_out : DEVICE, all N rows of H^l; only rows [dst_begin,dst_end) are written.
 * h_in and h_out must not overlap.  `workspace` is DEVICE scratch of at least
 * dgi_layer_workspace_bytes(...) bytes, 256-byte aligned, contents undefined before and after.
 * A transform-first layer needs the transformed rows of every source node, so it transforms all N
 * rows on every call: use dgi_infer, which does that once per layer, when running many batches.
 * Fast paths need 16-byte aligned rows (pointer and ld*elemsize multiples of 16); other layouts are
 * accepted and run on a slower element-wise gather.  An empty range, or N == 0, returns DGI_OK. */
dgi_status_t dgi_layer_forward(const dgi_graph_t* g, const dgi_layer_t* layer, const void* h_in, int64_t ld_in,
                               void* h_out, int64_t ld_out, int64_t dst_begin, int64_t dst_end,
                               void* workspace, uint64_t workspace_bytes, void* hip_stream);
dgi_status_t dgi_layer_workspace_bytes(const dgi_graph_t* g, const dgi_layer_t* layer, int64_t dst_begin,
                                       int64_t dst_end, uint64_t* bytes /*HOST*/);

/* dgi_layer_forward for callers that can neither allocate device memory nor pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and kernels as
 * dgi_layer_forward, but the workspace is a static device array of DGI_STATIC_WORKSPACE_BYTES bytes that is part of
 * the library's code object (every GPU the library runs on holds one copy until the process ends).  The call
 * allocates and frees nothing, on the device or through any library.  A layer / row range whose
 * dgi_layer_workspace_bytes exceeds DGI_STATIC_WORKSPACE_BYTES is refused with DGI_ERR_UNSUPPORTED (a transform-first
 * layer needs the transformed rows of all N nodes in the workspace, so this bounds N for those).  The calling thread's
 * current device must be the graph's.  All calls on one GPU share the one array and it keeps the previous call's
 * contents (every region is rewritten before it is read): calls that overlap in time on one GPU, on any streams,
 * race; order them on one stream or with events. */
#define DGI_STATIC_WORKSPACE_BYTES (32u << 20)
dgi_status_t dgi_layer_forward_static(const dgi_graph_t* g, const dgi_layer_t* layer, const void* h_in, int64_t ld_in,
                                      void* h_out, int64_t ld_out, int64_t dst_begin, int64_t dst_end, void* hip_stream);

/* Whole-model layer-wise inference (Algorithm 2): for l = 1..L, for every batch of destination rows,
 * compute H^l[batch]; H^{l-1} is released when layer l is done (two ping-pong buffers).
 *   x   : DEVICE [N x layers[0].in_dim], dtype layers[0].feat_dtype, leading dimension ld_x.
 *   out : DEVICE [N x layers[L-1].out_dim], dtype layers[L-1].out_dtype, leading dimension ld_out.
 *   layers[l].in_dim must equal layers[l-1].out_dim and feat_dtype must equal the previous out_dtype.
 * The call takes its hidden buffers and temporaries (Algorithm 2's H^l and per-batch buffers) from one
 * arena within opts->mem_budget_bytes.  The arena is allocated with hipMalloc on the first call, kept in
 * the graph handle and reused by later calls (reallocated when a call needs more, or when it is larger than
 * the call's budget); dgi_graph_release_workspace or dgi_graph_free returns it.  Calls on one graph handle
 * are serialised by a lock.  The call waits for its work on the stream before returning.
 * opts may be NULL (all defaults). */
dgi_status_t dgi_infer(const dgi_graph_t* g, const dgi_layer_t* layers, int32_t num_layers, const void* x,
                       int64_t ld_x, void* out, int64_t ld_out, const dgi_infer_opts_t* opts, void* hip_stream);

/* Partial inference (Sections 2 and 3.3): output embeddings of `num_targets` target nodes only.
 *   targets : DEVICE, int32 node ids (duplicates allowed);  out: DEVICE [num_targets x out_dim], row i = target i.
 * The per-layer target sets V^L = targets, V^{l-1} = V^l + in-neighbours(V^l) are marked on the device, and layer l
 * computes the rows of V^l only.  When |V^l| * average degree >= num_nodes the sets below V^l are taken to be all
 * nodes (the paper's shortcut): layers 1 .. l-1 run on the whole graph with dgi_infer, and only the inputs of layer l
 * are marked exactly.  The remaining layers run on a relabelled sub-problem (the rows of the first of them with their
 * complete in-neighbour lists, its inputs, nodes numbered by descending depth so that every V^l is a range of ids)
 * with the ordinary layer-wise schedule; degrees in the GCN normaliser remain those of the full graph.  When the
 * sub-problem would hold half of the graph's nodes or more, all layers run on the whole graph instead.
 * opts->perm_new_of_old must be NULL.  Waits for completion.  pstats (HOST, may be NULL) reports the set sizes. */
typedef struct {
    int32_t num_layers;
    int32_t all_nodes_from_layer;            /* l >= 1: layers 1 .. l ran on all nodes (shortcut; l = num_layers when the marked
                                                input set was half of the graph or more and nothing was extracted); -1: none */
    int64_t set_size[DGI_MAX_LAYERS + 1];    /* |V^l| for the annotated layers, index l in [0, num_layers] */
    int64_t sub_nodes, sub_edges;            /* size of the sub-problem that was extracted */
    int64_t rows_computed[DGI_MAX_LAYERS];   /* destination rows layer l (0-based) computed: |V^{l+1}|, or N under the shortcut */
} dgi_partial_stats_t;
dgi_status_t dgi_infer_partial(const dgi_graph_t* g, const dgi_layer_t* layers, int32_t num_layers, const void* x,
                               int64_t ld_x, const int32_t* targets, int64_t num_targets, void* out, int64_t ld_out,
                               const dgi_infer_opts_t* opts, dgi_partial_stats_t* pstats, void* hip_stream);

/* Layer-wise inference with the embeddings outside the GPU (Algorithm 2 as Sections 2 and 4.1 describe it:
 * the graph structure is on the device, the feature matrices H^0 .. H^L live in host memory, and every batch
 * loads its input set, computes one layer for its destination rows and dumps them back).
 *   x_host   : HOST, page-locked (hipHostMalloc / a pinned tensor), [N x layers[0].in_dim], leading dimension ld_x.
 *   out_host : HOST, page-locked, [N x layers[L-1].out_dim], leading dimension ld_out; only columns [0, out_dim) of
 *              its rows are written.
 * Hidden layers H^1 .. H^{L-1} are kept in two page-locked host buffers used alternately (H^{l-1}'s buffer is
 * reused when layer l is done); they and the device memory of the batches stay in the graph handle between
 * calls (dgi_graph_release_workspace or dgi_graph_free returns them), and calls on one handle are serialised.
 * Per batch [b, e) of destination rows the device (i) marks and compacts the input set I = [b, e) + the sources of the batch's edges, (ii) reads the rows H^{l-1}[I] straight
 * from host memory into a compact device matrix, (iii) relabels the batch's neighbour lists to positions in I
 * and runs the layer (dgi_layer_forward's kernels) on that sub-problem, (iv) copies the rows H^l[b:e] to host.
 * Up to two batches are in flight: while one computes and dumps on a second stream, the next one is built and loaded
 * (the host link carries both directions at once); a batch may then use M = half of opts->mem_budget_bytes
 * (0 = 90 % of free device memory).  Smaller batches load more rows in total, so the library runs one batch at a
 * time with M = the whole budget instead whenever it estimates, on the first planned batch, that compute and
 * dump are a small part of a batch's time next to its load (hstats->slots tells which).  Batch sizes follow Section 4.1 with real memory at stake: the batch's
 * device memory M_k (input rows, relabelled lists, output rows, layer workspace) is measured, the thresholds are
 * rescaled by r = M / M_k (Eq. 2), and a batch that does not fit M halves the thresholds and is planned again.
 * A layer that multiplies before it aggregates (out_dim < in_dim, GAT) and whose transformed rows are at most
 * three quarters as wide as its input rows runs as two passes when it needs more than one batch: H^{l-1} streams
 * through the device once in contiguous row chunks and Z = H^{l-1} W goes to a page-locked buffer, then the
 * batches load rows of Z for their input sets and only aggregate (input_bytes counts rows of Z, transform_bytes
 * the dense pass).  For GraphSAGE the batches load only the z_neigh block of those rows (that block's width is what
 * the three-quarters rule compares) plus the z_self block of their own destination rows, a contiguous run.
 * When the whole graph fits M, every layer is one batch; when x, the output and dgi_infer's own buffers all fit
 * the budget, the call is one copy in, dgi_infer, one copy out (hstats->device_resident = 1) and the hidden
 * layers never leave the device (opts->host_stream_always = 1 switches that off).  opts->batch_size > 0 fixes
 * the rows per batch instead;
 * opts->perm_new_of_old and opts->jk_concat are not supported here, opts->stats is ignored.
 * Waits for completion.  hstats (HOST, may be NULL) reports what was moved. */
typedef struct {
    int32_t num_layers;
    int32_t device_resident;                 /* 1: everything fitted the budget, the hidden layers never left the device */
    double  total_ms;                        /* wall-clock of the call */
    double  load_ms[DGI_MAX_LAYERS];         /* input-set construction + rows read from host memory */
    double  compute_ms[DGI_MAX_LAYERS];      /* the layer's kernels */
    double  store_ms[DGI_MAX_LAYERS];        /* rows copied back to host memory */
    int64_t batches[DGI_MAX_LAYERS];
    int64_t input_rows[DGI_MAX_LAYERS];      /* sum over batches of |I| (what node reordering shrinks, Section 4.2) */
    int64_t input_bytes[DGI_MAX_LAYERS];     /* bytes read from host memory */
    int64_t output_bytes[DGI_MAX_LAYERS];    /* bytes written to host memory */
    int64_t transform_bytes[DGI_MAX_LAYERS]; /* dense pass of a transform-first layer: rows of H^{l-1} read + rows of Z written */
    int64_t oom_retries;                     /* batches planned again after halving the thresholds */
    int64_t peak_batch_bytes;                /* largest M_k */
    int64_t budget_bytes;                    /* M, the memory one batch may use */
    int64_t slots;                           /* batches in flight: 1 or 2 (0 when device_resident) */
} dgi_host_stats_t;
dgi_status_t dgi_infer_host(const dgi_graph_t* g, const dgi_layer_t* layers, int32_t num_layers, const void* x_host,
                            int64_t ld_x, void* out_host, int64_t ld_out, const dgi_infer_opts_t* opts,
                            dgi_host_stats_t* hstats, void* hip_stream);

/* Sampling inference (Section 2: each node aggregates a sampled subset of its in-neighbours; the paper's
 * experiments use a fan-out of 10 for all layers).
 * dgi_graph_sample: the sampled graph of layer `layer` as a new handle (free it with dgi_graph_free).  A row with
 * at most `fanout` in-edges keeps them all; otherwise it keeps the `fanout` edges with the smallest keys, in stored
 * order, a uniform sample without replacement.  The key of the edge at position e of `indices` is the upper 32
 * bits of output number layer*E + e + 1 of the SplitMix64 generator seeded with `seed` (equal keys ordered by
 * position in the row), so the sample is a pure function of (graph, fanout, seed, layer).  Waits for completion.
 * dgi_infer_sampled: layer l of the model runs on dgi_graph_sample(g, fanout, seed, l) with the ordinary
 * layer-wise schedule (dgi_infer on one layer; opts as there, perm_new_of_old / jk_concat / stats unsupported);
 * the mean and GCN normalisers use the degrees of the sampled graph.  x, out: DEVICE, as for dgi_infer.  The
 * hidden layers, the schedule's arena, the sample's indptr (it depends on the degrees and the fan-out only, so it is
 * computed once per fan-out) and the sampler's buffers are kept in g's handle between calls
 * (dgi_graph_release_workspace returns them); calls on one handle are serialised.  Waits for completion. */
dgi_status_t dgi_graph_sample(const dgi_graph_t* g, int32_t fanout, uint64_t seed, int32_t layer, void* hip_stream,
                              dgi_graph_t** g_out);
dgi_status_t dgi_infer_sampled(const dgi_graph_t* g, const dgi_layer_t* layers, int32_t num_layers, const void* x,
                               int64_t ld_x, void* out, int64_t ld_out, int32_t fanout, uint64_t seed,
                               const dgi_infer_opts_t* opts, void* hip_stream);

/* ------------------------------------------------------------------------------------------------
 * Host-side planning helpers (no device access; usable without a GPU).
 *
 * dgi_plan_batch_end: the batching rule of Section 4.1.  The in-degree prefix sum is `indptr` itself;
 * starting at row `begin`, returns by binary search the largest `end` <= row_limit with
 * end-begin <= n_t and indptr[end]-indptr[begin] <= n_i, but never less than begin+1 (a row whose own
 * degree exceeds n_i forms a batch by itself).  indptr is a HOST array. */
dgi_status_t dgi_plan_batch_end(const void* indptr, int32_t indptr_type, int64_t row_limit, int64_t begin,
                                int64_t n_t, int64_t n_i, int64_t* end);
/* Eq. 2: r = M / M_k; n_t <- r n_t; n_i <- r n_i (both kept >= 1).  M_k <= 0 leaves them unchanged. */
dgi_status_t dgi_threshold_update(double M_expected, double M_k, int64_t* n_t, int64_t* n_i);
/* Out-of-memory reaction of Section 4.1: halve both thresholds (floor, >= 1).  Returns DGI_ERR_OOM when
 * both are already 1. */
dgi_status_t dgi_threshold_halve(int64_t* n_t, int64_t* n_i);
/* Number of distinct source nodes the batch [begin,end) reads (the "input set" of Section 4.2's example);
 * HOST CSR, indptr as int64. */
dgi_status_t dgi_batch_input_set_size(int64_t num_nodes, const int64_t* indptr, const int32_t* indices,
                                      int64_t begin, int64_t end, int64_t* count);
/* The permutation dgi_graph_reorder would use, computed from a HOST CSR (indptr int64). */
dgi_status_t dgi_reorder_permutation(int64_t num_nodes, const int64_t* indptr, const int32_t* indices,
                                     int32_t method, uint64_t seed, int32_t* perm_new_of_old);

/* Page-locked host memory of exactly `bytes` bytes for dgi_infer_host's x_host / out_host (hipHostMalloc; any other
 * page-locked allocation serves as well — this pair exists for callers whose framework's pinned allocator rounds
 * sizes up, which at tens of gigabytes decides whether the matrices of Algorithm 2 fit the lockable memory).
 * dgi_host_free(NULL) is a no-op. */
dgi_status_t dgi_host_alloc(uint64_t bytes, void** ptr);
dgi_status_t dgi_host_free(void* ptr);

const char* dgi_status_string(dgi_status_t s);
const char* dgi_last_error(void);  /* thread-local, never NULL */
int32_t     dgi_version(void);     /* major*1000 + minor */

#ifdef __cplusplus
}
#endif
#endif /* DGI_H */
