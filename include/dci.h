/*
 * dci.h - C boundary of the MI355X (gfx950) implementation of the dual-cache GNN inference
 * hot path of DCI (arXiv 2503.01281): pre-sampling access counting, the workload-aware
 * dual-cache fill, cache-aware multi-hop neighbour sampling, cache-aware feature gathering
 * and the forward pass (GraphSAGE with the mean aggregator; the sum-aggregate GraphSAGE and the
 * averaging GCN of the paper's Table III through dci_gnn_forward).
 *
 * General rules
 *  - C linkage, plain pointers and sizes.  Every call returns a status (0 = DCI_OK, negative =
 *    error) and never throws or aborts; dci_last_error() gives the message of the last failure
 *    on that context.
 *  - The caller owns every buffer.  "device" pointers are HBM allocations on the context's GPU.
 *    "mapped" pointers may be HBM or pinned host memory that the GPU can dereference
 *    (hipHostMalloc / a pinned PyTorch tensor): the graph and the feature matrix normally live
 *    there and are read by zero-copy on a cache miss (Section IV, framework paragraph).
 *  - The library allocates no device memory.  Temporary device memory comes from the workspace
 *    handed to dci_create(); the dci_*_workspace_bytes() queries say how much each call needs.
 *    (A context owns a few HIP events and 64 bytes of pinned host memory; dci_timing_enable
 *    creates events on first use.)
 *  - Calls enqueue work on the context's HIP stream and return without waiting, except
 *    dci_fill_caches(), which waits for completion because the cache sizes it reports are
 *    computed on the GPU.  Device outputs, and host outputs marked "valid after dci_sync", may be
 *    read after dci_sync() (or any synchronisation of that stream).  Calls on one context must
 *    not overlap in time on different host threads.
 *  - Node ids are int64 (global) or int32 (local to a mini-batch), counters are uint32,
 *    features and weights are fp32, row-major.
 *  - Fan-outs are given in execution order, from the seed nodes outward (the paper prints them
 *    in layer order, e.g. "15,10,5" = fan-outs {5,10,15} here).
 */
#ifndef DCI_H_
#define DCI_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DCI_MAX_HOPS 8
#define DCI_MAX_FANOUT 64

#define DCI_OK 0
#define DCI_ERR_INVALID_ARG (-1) /* NULL pointer, negative size, fan-out out of range, ...          */
#define DCI_ERR_CAPACITY (-2)    /* a caller buffer or the workspace is too small (see message)      */
#define DCI_ERR_HIP (-3)         /* a HIP runtime call failed                                        */
#define DCI_ERR_UNSUPPORTED (-4) /* a size beyond what the kernels index (e.g. more than 2^31 nodes) */

#define DCI_FEAT_POLICY_PAPER_MEAN 0 /* above-average nodes first, then the rest (Section IV-B)     */
#define DCI_FEAT_POLICY_TOPK 1       /* nodes by visit count, descending                            */
#define DCI_FILL_STRICT_SPLIT 0x100  /* OR-ed into feat_policy: keep the shares of Eq. (1) as they
                                        are, no spill-over; with t_sample_ns = 0 this is the
                                        single-cache system of Section V-B (no adjacency cache)    */
#define DCI_FILL_ADJ_ELEMENTS 0x200  /* OR-ed into feat_policy: element-granular adjacency cache, i.e.
                                        Algorithm 1 with its second-level sort and a last node that
                                        may be cached in part; needs edge_count and rewrites
                                        graph->indices in place (see dci_fill_caches)              */

typedef struct dci_ctx dci_ctx;

/* The graph and its features (Section II-C).  The adjacency structure is the compressed
 * sparse column form of the paper with the target node as the column: the in-neighbours of
 * node v are indices[indptr[v] .. indptr[v+1]).  Unweighted, so there is no Values array. */
typedef struct {
  int64_t num_nodes;      /* N, 1 .. 2^31-1                                   */
  int64_t num_edges;      /* E = indptr[N]                                    */
  int32_t feat_dim;       /* F >= 1                                           */
  const int64_t* indptr;  /* [N+1] mapped, borrowed                           */
  const int64_t* indices; /* [E]   mapped, borrowed                           */
  const float* feat;      /* [N,F] mapped, borrowed (may be NULL for sampling-only calls) */
} dci_graph;

/* The dual cache (Section IV).  Filled by dci_fill_caches(); all pointers are device memory.
 * A NULL dci_cache* argument means "no cache": every access takes the miss path. */
typedef struct {
  int64_t adj_nodes;      /* K: nodes whose neighbour lists are cached                  */
  int64_t adj_edges;      /* M: cached list elements                                    */
  int64_t feat_rows;      /* k: cached feature rows                                     */
  uint64_t adj_bytes;     /* 8*(K+1) + 8*M                                              */
  uint64_t feat_bytes;    /* 4*F*k                                                      */
  uint64_t cap_adj_bytes; /* C_adj of Eq. (1) after spill-over                          */
  uint64_t cap_feat_bytes;/* C_feat of Eq. (1) after spill-over                         */
  const int32_t* adj_remap;  /* [N] slot in the adjacency cache, or -1                  */
  const int64_t* c_indptr;   /* [K+1]                                                   */
  const int64_t* c_indices;  /* [M] the cached lists, in the order the host lists have  */
  int64_t adj_partial_node;  /* the one node whose list is cached only in its leading part
                                (element-granular fill), or -1; counted in K               */
  int64_t adj_partial_deg;   /* its full list length (the cached length is in c_indptr)    */
  const int32_t* feat_remap; /* [N] row in the feature cache, or -1                     */
  const float* feat_cache;   /* [k,F]                                                   */
} dci_cache;

/* One sampled mini-batch: L bipartite blocks and the node lists F_0 (seeds) .. F_L (input
 * nodes).  F_h is the prefix of `nodes` of length n_nodes[h]; F_{h+1} is F_h followed by the
 * nodes first reached at hop h, in the order of their first appearance over the hop's edges
 * taken row by row.  Block h has one row per node of F_h; row i holds the local ids (indices
 * into F_{h+1}) of the neighbours sampled for F_h[i].
 * All arrays are caller-allocated device memory with at least the capacities that
 * dci_blocks_bounds() returns for the call's (n_seeds, fanouts).  The sizes of the batch are
 * produced on the GPU, in `counts`: n_nodes[h] = counts[h] (h = 0..L) and
 * n_edges[h] = counts[DCI_MAX_HOPS + 1 + h]; later calls read them there, so a pipeline needs
 * no host round trip.  counts_host (nullable, pinned host memory of the same shape) receives a
 * copy that is valid after dci_sync. */
typedef struct {
  int32_t n_hops;
  int64_t cap_nodes;                 /* entries in nodes[]                                */
  int64_t cap_rows[DCI_MAX_HOPS];    /* blk_indptr[h] has cap_rows[h] + 1 entries         */
  int64_t cap_edges[DCI_MAX_HOPS];   /* entries in blk_src[h]                             */
  int64_t* nodes;                    /* device [cap_nodes] global ids                     */
  int64_t* blk_indptr[DCI_MAX_HOPS]; /* device                                            */
  int32_t* blk_src[DCI_MAX_HOPS];    /* device                                            */
  int64_t* counts;                   /* device [2*DCI_MAX_HOPS + 1]                       */
  int64_t* counts_host;              /* pinned host [2*DCI_MAX_HOPS + 1] or NULL          */
} dci_blocks;

/* Per-call statistics, accumulated (+=) by the kernels into a caller-owned device array of
 * DCI_STATS_WORDS uint64 (clear it before the first use; copy it out after dci_sync).  Pass NULL
 * to skip them. */
enum {
  DCI_STAT_EDGES_SAMPLED = 0,  /* sampled edges over all hops                              */
  DCI_STAT_ADJ_NODE_HITS = 1,  /* frontier nodes whose list was in the adjacency cache     */
  DCI_STAT_ADJ_NODE_MISSES = 2,
  DCI_STAT_ADJ_EDGE_HITS = 3,  /* sampled edges read from the adjacency cache              */
  DCI_STAT_ADJ_EDGE_MISSES = 4,
  DCI_STAT_FEAT_HITS = 5,      /* gathered rows read from the feature cache                */
  DCI_STAT_FEAT_MISSES = 6,
  DCI_STAT_INPUT_NODES = 7,    /* sum of |F_L| over sampled batches                        */
  DCI_STAT_T_SAMPLE_NS = 8,    /* dci_presample_count only: GPU time spent sampling        */
  DCI_STAT_T_FEATURE_NS = 9,   /* dci_presample_count only: GPU time spent loading features */
  DCI_STAT_BYTES_HBM = 10,     /* bytes the caches served: 16 per frontier node with a slot (its pair of
                                  list bounds), 8 per edge read from the adjacency cache, 4F per row read
                                  from the feature cache                                              */
  DCI_STAT_BYTES_HOST = 11,    /* the same quantities for what the graph arrays served (the miss path) */
  DCI_STAT_LINES_BOUNDS = 12,  /* sampling misses: 128-byte lines of graph->indptr that the list bounds of
                                  the missed frontier nodes lie in (one or two per node), summed.  A node's
                                  bounds cross the link once per batch, at the hop at which the node joins
                                  the frontier: later hops, which sample it again, take them from a note
                                  the sampler keeps in HBM for the batch (the byte counters above still
                                  charge them to the tier that holds the node's list, hop by hop)        */
  DCI_STAT_LINES_IDS = 13,     /* sampling misses: distinct 128-byte lines of graph->indices read per
                                  frontier node, summed.  A host link charges a small read a whole
                                  request, so lines - not bytes - are what the miss path costs          */
  DCI_STAT_ROWS_COPIED = 14,   /* rows the gather wrote to its output: all of them for dci_gather_features,
                                  the misses and the rows of F_{L-1} for dci_gather_forward             */
  DCI_STATS_WORDS = 16
};

/* ---- context ----------------------------------------------------------------------------- */

/* Creates a context bound to GPU `device` and to `hip_stream` (a hipStream_t, borrowed; NULL =
 * the default stream).  `workspace` is device memory of `workspace_bytes` bytes, 256-byte
 * aligned, borrowed until dci_destroy; it may be NULL/0 and replaced later with
 * dci_set_workspace.  Returns DCI_ERR_HIP if the device cannot be selected. */
int32_t dci_create(dci_ctx** out, int32_t device, void* hip_stream, void* workspace, size_t workspace_bytes);
int32_t dci_set_workspace(dci_ctx* ctx, void* workspace, size_t workspace_bytes);
void dci_destroy(dci_ctx* ctx);
/* Waits for everything enqueued on the context's stream. */
int32_t dci_sync(dci_ctx* ctx);
/* Message of the last failed call on this context (never NULL; "" if none). */
const char* dci_last_error(const dci_ctx* ctx);

/* The sizes that the last dci_sample_khop / dci_sample_khop_static call on this context needed,
 * for a caller that got DCI_ERR_CAPACITY and wants to grow its buffers: cap_nodes[DCI_MAX_HOPS + 1]
 * (entries of blocks.nodes = cap_nodes[n_hops]; rows of block h = cap_nodes[h]), cap_edges[DCI_MAX_HOPS]
 * and the bytes of temporaries (workspace or static scratch).  Any pointer may be NULL.  The same
 * numbers come from dci_blocks_bounds and the *_workspace_bytes queries before a call. */
int32_t dci_last_required(const dci_ctx* ctx, int64_t* cap_nodes, int64_t* cap_edges, size_t* workspace_bytes);

/* Tuning options of a context.  None changes what is computed (the dense-layer kernels differ only
 * in the order of the floating-point sums).  DCI_ERR_INVALID_ARG for an unknown option or value.
 *   DCI_OPT_LINEAR_KERNEL  which dense-layer kernel dci_sage_forward / dci_gnn_forward launch:
 *       0  by shape (default): the kernel that keeps the weights in registers when the whole contraction
 *          is at most 256 long (two operands of up to 128 columns, or GCN's one of up to 256), the input width
 *          a multiple of 4, the output width a multiple of 256 and the layer at least 98304 rows tall by
 *          capacity; else the wide kernel (128-column tiles, one workgroup per compute unit)
 *          when the layer is at least 16384 rows tall by capacity, its input width is even and
 *          at least 192, its output width is a multiple of 128 and the operands are suitably
 *          aligned; else a 64x64 tile kernel, fed by global->LDS loads where the output width is a multiple of 64, the
 *          input width even and the contraction not split, through registers otherwise
 *       1  always the 64x64 tile kernel that stages its operands through registers
 *       2  the wide kernel whenever width and alignment allow it, whatever the row count
 *       3  like 0 without the wide and the weights-in-registers kernels
 *       4  the weights-in-registers kernel whenever widths and alignment allow it, whatever the row count;
 *          other layers as under 1 */
#define DCI_OPT_LINEAR_KERNEL 1
/*   DCI_OPT_LINEAR_SPLIT   upper limit on the workgroups that share one output tile of the 64x64 kernel
 *       (the contraction is split between them and a second kernel adds the partial sums in a fixed order):
 *       0  by shape (default): layers with few tiles are split up to 8 ways;  1  never split;  n <= 8  at most n */
#define DCI_OPT_LINEAR_SPLIT 2
/*   DCI_OPT_RELABEL_SPIN_LIMIT  how often a tile of the frontier scan (dedup + relabel, one chained prefix
 *       sum per hop) polls for its predecessors before it gives up; default 2^24, far beyond any real wait.
 *       A tile that gives up voids its batch: the remaining kernels of the batch do nothing, the batch's
 *       `counts` (and counts_host) are zeroed so that a following gather / forward finds no rows, and the
 *       next dci_sync (or dci_timing_read, or the waiting dci_presample_count) on the context returns
 *       DCI_ERR_HIP with the message "relabel scan timed out ...".  Pre-sampling counters updated by a
 *       voided batch are unspecified. */
#define DCI_OPT_RELABEL_SPIN_LIMIT 3
/*   DCI_OPT_TEST_RELABEL_FIRST_TICKET  test hook for that failure path, off (0) by default: the scan numbers
 *       its tiles from this value, so the tiles below it never run or publish and the first real tile must
 *       give up.  Only accepted while the spin limit is at most 65536, so that every kernel still ends
 *       within microseconds. */
#define DCI_OPT_TEST_RELABEL_FIRST_TICKET 4
/*   DCI_OPT_FUSED_INPUT  how dci_infer_batches feeds the model on this context's lane: 0 (default)
 *       dci_gather_features then dci_gnn_forward, so that the lane's x holds every gathered row;
 *       1 dci_gather_forward (cached neighbour rows are read in place; x holds only the rows that
 *       missed and those of F_{L-1}).  The logits are bit-identical either way: the sums run in the same order. */
#define DCI_OPT_FUSED_INPUT 5
/*   DCI_OPT_RELABEL_TILE_ITERS  rows per lane group in a tile of the frontier scan: 0 (default) chosen from
 *       the frontier's size, or 2, 4, 8.  Tuning only: the result does not depend on it. */
#define DCI_OPT_RELABEL_TILE_ITERS 6
/*   DCI_OPT_INPUT_LAYER  how the forward pass runs its first layer (two operands of at most 128 columns, mean or
 *       sum aggregator).  There are two one-kernel forms that keep the aggregated rows out of device memory:
 *       "registers" - the aggregation runs inside the weights-in-registers dense kernel (needs what that kernel
 *       needs, see DCI_OPT_LINEAR_KERNEL) - and "tiles" - half of each workgroup aggregates 64 rows into LDS while
 *       the other half multiplies the 64 rows before (needs a width that is a multiple of 16, at least 32, an
 *       output width that is a multiple of 64, 16-byte aligned rows, weights, bias and output).
 *       0 (default): for layers of at least 98,304 rows (capacity) the registers form if the two operands together
 *       are at most 208 columns (13 slabs of 16: beyond that the weights leave too few registers for the loads in
 *       flight), else the tiles form if the shape allows it, else two kernels;  1: always the aggregation kernel
 *       followed by a dense kernel;  2: the registers form whenever widths and alignment allow it, whatever the
 *       row count;  3: the tiles form likewise.  The registers form is bit-identical to the two-kernel route; the
 *       tiles form is bit-identical to it where the contraction needs no padding (width a multiple of 16) and the
 *       two-kernel route ends in the weights-in-registers kernel, and within rounding of it otherwise. */
#define DCI_OPT_INPUT_LAYER 7
int32_t dci_set_option(dci_ctx* ctx, int32_t option, int64_t value);

/* Kernel timing, for benchmarks and profiles.  Kernel classes whose bit is set in class_mask are
 * bracketed by HIP events on the context's stream (up to DCI_TIMING_MAX_LAUNCHES launches
 * between two reads; later ones are not recorded).  dci_timing_read waits for the stream, adds
 * up the elapsed time and the number of recorded launches per class into total_ms[DCI_K_COUNT]
 * and launches[DCI_K_COUNT], and starts over.  class_mask = 0 switches timing off (the default). */
enum {
  DCI_K_TABLE_CLEAR = 0, /* clearing the batch's hash table and scan status words   */
  DCI_K_SAMPLE = 1,      /* per hop: draw positions, read neighbours, register ids
                            (also writes the previous hop's edge local ids)        */
  DCI_K_RELABEL = 2,     /* per hop: first appearances, row offsets, new local ids  */
  DCI_K_WRITE_SRC = 3,   /* last hop: local id of every edge, batch sizes to host   */
  DCI_K_GATHER = 4,      /* feature gather                                          */
  DCI_K_MEAN_IN = 5,     /* first layer (input features): neighbour mean            */
  DCI_K_LINEAR_IN = 6,   /* first layer (input features): dense layer (matrix cores) */
  DCI_K_MEAN = 7,        /* later layers: neighbour mean                            */
  DCI_K_LINEAR = 8,      /* later layers: dense layer                               */
  DCI_K_COUNT_NODES = 9, /* pre-sampling: visits of the input nodes                 */
  DCI_K_COUNT = 10
};
#define DCI_TIMING_MAX_LAUNCHES 8192
int32_t dci_timing_enable(dci_ctx* ctx, uint32_t class_mask);
int32_t dci_timing_read(dci_ctx* ctx, double* total_ms, int64_t* launches);

/* Memory-rate probe, for benchmarks: the rates that the access-bound steps are measured against
 * (Section IV, framework paragraph: a hit reads GPU memory, a miss reads host memory through the
 * zero-copy mapping).  Reads `mem` (device memory, or pinned host memory that the GPU can
 * dereference; 256-byte aligned, `bytes` >= 4096) on the context's stream, waits, and returns the
 * GPU time of the one kernel in *ms.
 *   granule = 0            streaming read of the whole region, 16 bytes per lane;
 *   granule = 8 .. 512     n_access reads of aligned `granule`-byte pieces at pseudo-random places
 *                          (8 and 16: one lane each; above: 16 bytes per lane, granule/16 lanes);
 *   granule = -64          64-byte pieces read as eight 8-byte words by eight lanes.
 *   order (granule != 0)   0: the lanes of a piece are adjacent and take its words in order;
 *                          1: adjacent lanes, words in a scrambled order; 2: the lanes of a piece
 *                          are spread over the wavefront (never adjacent).
 * workgroups (1..65536) of 256 lanes are launched; sink: device uint64 [workgroups], scratch. */
int32_t dci_probe_read(dci_ctx* ctx, const void* mem, uint64_t bytes, int32_t granule, int32_t order,
                       int64_t n_access, int32_t workgroups, uint64_t seed, uint64_t* sink, float* ms);

/* Upper bounds on the sizes of a mini-batch with n_seeds seeds: cap_nodes[h] bounds |F_h|
 * (h = 0..n_hops), cap_edges[h] the edges of block h.  |F_{h+1}| <= min(|F_h| (1 + f_h),
 * N + n_seeds).  Returns DCI_ERR_INVALID_ARG for n_hops outside 1..DCI_MAX_HOPS or a fan-out
 * outside 1..DCI_MAX_FANOUT, DCI_ERR_UNSUPPORTED if a bound reaches 2^31. */
int32_t dci_blocks_bounds(int64_t num_nodes, int64_t n_seeds, const int32_t* fanouts, int32_t n_hops,
                          int64_t* cap_nodes, int64_t* cap_edges);

/* Workspace needed by dci_sample_khop / dci_presample_count for batches of up to n_seeds seeds. */
size_t dci_sample_workspace_bytes(int64_t num_nodes, int64_t n_seeds, const int32_t* fanouts, int32_t n_hops);
/* Workspace needed by dci_fill_caches.  With DCI_FILL_ADJ_ELEMENTS it needs the larger
 * dci_fill_elements_workspace_bytes(num_nodes, n_elements), where n_elements bounds the total
 * list length of the nodes with a non-zero adj_count (num_edges always does; more than 2^31 - 1
 * such elements are not supported). */
size_t dci_fill_workspace_bytes(int64_t num_nodes);
size_t dci_fill_elements_workspace_bytes(int64_t num_nodes, int64_t n_elements);
/* Workspace needed by dci_sage_forward for blocks with these row capacities. */
size_t dci_sage_workspace_bytes(const int64_t* cap_rows, int32_t n_layers, const int32_t* dims);

/* ---- the five calls of the hot path ------------------------------------------------------- */

/* Pre-sampling access counting (Section IV-A, first paragraph; Section IV-B, first paragraph).
 * Samples the batches [first_batch, first_batch + n_batches) of the seed list - batch b covers
 * seeds[b*batch_size .. min(n_seeds, (b+1)*batch_size)) and uses RNG batch index
 * rng_batch0 + (b - first_batch) - exactly as dci_sample_khop would, and accumulates
 *   adj_count[v]  += 1 and edge_count[indptr[v] + p] += 1 for every sampled position p of every
 *                    frontier node v at every hop,
 *   feat_count[u] += 1 for every node u of each batch's input list F_L.
 * feat_count, adj_count: device uint32 [N]; edge_count: device uint32 [E] or NULL.  The
 * counters are not cleared.  If feat_scratch (device, >= cap_nodes[L] * F floats) is not NULL
 * each batch's input rows are also gathered into it, and the GPU times of the sampling part and
 * of the gathering part are added to DCI_STAT_T_SAMPLE_NS / DCI_STAT_T_FEATURE_NS (the two
 * times of Eq. (1)); this makes the call wait for the GPU.  cache may be NULL (the usual case:
 * nothing is cached yet).  seeds: device int64 [n_seeds], distinct. */
int32_t dci_presample_count(dci_ctx* ctx, const dci_graph* graph, const dci_cache* cache,
                            const int64_t* seeds, int64_t n_seeds, int32_t batch_size, int64_t first_batch,
                            int64_t n_batches, uint64_t rng_batch0, const int32_t* fanouts, int32_t n_hops,
                            uint64_t rng_seed, uint32_t* feat_count, uint32_t* adj_count,
                            uint32_t* edge_count, float* feat_scratch, uint64_t* stats);

/* Capacity split and dual-cache fill (Eq. (1); Section IV-B; Algorithm 1).
 *  1. C_adj = floor(budget * t_sample / (t_sample + t_feature)), C_feat = budget - C_adj
 *     (half each when both times are 0).  A share larger than its side can use - the whole
 *     adjacency structure is 8*(N+1+E) bytes, the whole feature matrix 4*N*F - is cut to that
 *     and the excess moves to the other side, so a budget that covers the dataset caches all
 *     of it (unless DCI_FILL_STRICT_SPLIT is set in feat_policy).
 *  2. Feature cache: k = min(N, C_feat / (4F)) rows.  DCI_FEAT_POLICY_PAPER_MEAN takes the nodes
 *     whose feat_count exceeds the mean over all N nodes, in ascending id, then the other nodes
 *     in ascending id, and keeps the first k.  DCI_FEAT_POLICY_TOPK orders by feat_count
 *     descending (ties: ascending id).  feat_remap[v] = row or -1.
 *  3. Adjacency cache: if 8*(N+1+E) <= C_adj the whole structure is cached with slot = node id.
 *     Otherwise nodes are ordered by adj_count descending (ties: ascending id) and the longest
 *     prefix whose compacted form 8*(K+1) + 8*sum(deg) fits in C_adj is cached, lists
 *     concatenated in that order, each in its original element order.  adj_remap[v] = slot or -1.
 *     With DCI_FILL_ADJ_ELEMENTS (Algorithm 1 and Fig. 6 as printed) the second branch also
 *     reorders the elements inside every node by their own edge_count descending (ties: original
 *     order), in graph->indices itself, so that position p of a list means the same neighbour in
 *     the cache and on the host.  Because this rewrites an array the graph struct only lends as
 *     const, the caller must say so: indices_rw must then be the same address as graph->indices,
 *     writable mapped memory (DCI_ERR_INVALID_ARG otherwise; ignored, and may be NULL, without the
 *     flag).  Everything else that holds this graph - other contexts, caches filled earlier,
 *     per-element counters - refers to the old order afterwards.  And the
 *     first node that does not fit as a whole is cached in part when at least 16 bytes are left:
 *     its pointer entry and its floor((left - 8) / 8) leading elements (adj_partial_node /
 *     adj_partial_deg).  A sampled position p of a node with a slot is served by the cache iff
 *     p < cached length.  adj_count[v] must be the sum of edge_count over v's list (as
 *     dci_presample_count leaves them); edge_count (device uint32 [E]) is not modified but no
 *     longer matches the reordered lists afterwards.  The mode needs additional workspace, see
 *     dci_fill_elements_workspace_bytes().
 * cache_buf: device, 256-byte aligned, at least budget_bytes + 256 bytes; the cache arrays are
 * carved from it (feature rows first).  adj_remap, feat_remap: device int32 [N], written in
 * full.  edge_count is only read with DCI_FILL_ADJ_ELEMENTS (may be NULL otherwise).  *out is
 * filled on return; this call waits for the GPU. */
int32_t dci_fill_caches(dci_ctx* ctx, const dci_graph* graph, const uint32_t* feat_count,
                        const uint32_t* adj_count, const uint32_t* edge_count, uint64_t budget_bytes,
                        uint64_t t_sample_ns, uint64_t t_feature_ns, int32_t feat_policy, void* cache_buf,
                        int32_t* adj_remap, int32_t* feat_remap, int64_t* indices_rw, dci_cache* out);

/* Cache-aware multi-hop uniform neighbour sampling (Section II-C; Section IV, framework
 * paragraph; hit rule of Section IV-B, third paragraph).
 * For hop h and every node v = F_h[i]: deg = length of v's list, c = min(fanouts[h], deg).
 * deg <= fanout takes the whole list in order; otherwise Floyd's subset algorithm draws c
 * distinct positions, slot s using the Philox4x32-10 output for key = rng_seed and counter =
 * (v lo, v hi, batch_index, h << 24 | s), reduced to [0, deg - c + s] by a 64x64 -> high-64
 * multiply.  The list (and its length) is read from the adjacency cache when
 * cache->adj_remap[v] >= 0 and from graph->indptr/indices otherwise; both hold the same bytes,
 * so the result does not depend on the cache.  seeds: device int64 [n_seeds]; duplicates are
 * tolerated (they share a local id).  batch_index < 2^32.  out: see dci_blocks. */
int32_t dci_sample_khop(dci_ctx* ctx, const dci_graph* graph, const dci_cache* cache, const int64_t* seeds,
                        int64_t n_seeds, uint64_t batch_index, const int32_t* fanouts, int32_t n_hops,
                        uint64_t rng_seed, dci_blocks* out, uint64_t* stats);

/* dci_sample_khop for callers that cannot allocate device memory or hand over a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernels and the same result as dci_sample_khop, but the temporaries (hash table, scan status
 * words, padded per-hop arrays) live in an array of DCI_STATIC_SCRATCH_BYTES bytes that is part of
 * the library's device code: every GPU the library runs on holds its own copy until the process
 * ends, and the context's workspace is neither needed nor touched.  The call allocates nothing.
 * A batch whose bounds need more than the array holds - dci_sample_khop_scratch_bytes(num_nodes,
 * n_seeds, fanouts, n_hops) says how much a call needs (0 for invalid arguments) - is rejected with
 * DCI_ERR_CAPACITY and a message naming both sizes.  All contexts on one GPU share that GPU's array
 * and a call leaves its temporaries behind (every call clears what it needs cleared itself): two
 * calls that overlap in time on one GPU, on whatever streams or contexts, race. */
#define DCI_STATIC_SCRATCH_BYTES (32u << 20)
int32_t dci_sample_khop_static(dci_ctx* ctx, const dci_graph* graph, const dci_cache* cache,
                               const int64_t* seeds, int64_t n_seeds, uint64_t batch_index,
                               const int32_t* fanouts, int32_t n_hops, uint64_t rng_seed, dci_blocks* out,
                               uint64_t* stats);
size_t dci_sample_khop_scratch_bytes(int64_t num_nodes, int64_t n_seeds, const int32_t* fanouts,
                                     int32_t n_hops);

/* Cache-aware feature gather (Section IV, framework paragraph; Section IV-B, first paragraph):
 * out[i,:] = feat_cache[feat_remap[id_i],:] on a hit, graph->feat[id_i,:] on a miss.
 * node_ids: device int64.  The number of rows is *n_dev (device int64, e.g. &counts[L] of a
 * dci_blocks) when n_dev is not NULL, with n_max an upper bound used to size the launch;
 * otherwise it is n_max.  out: device [n_max, F]. */
int32_t dci_gather_features(dci_ctx* ctx, const dci_graph* graph, const dci_cache* cache,
                            const int64_t* node_ids, int64_t n_max, const int64_t* n_dev, float* out,
                            uint64_t* stats);

/* GraphSAGE-mean forward over the blocks of one mini-batch (Table III family; mean aggregator).
 * Layer l = 0..n_layers-1 works on block h = n_layers-1-l: for each row i < n_nodes[h]
 *   m_i = mean of x[src] over the row's edges (zero vector for an empty row)
 *   y_i = x_i W_self[l] + m_i W_neigh[l] + bias[l], ReLU on all layers but the last.
 * x_in: device [n_nodes[L], dims[0]]; w_self[l], w_neigh[l]: device [dims[l], dims[l+1]]
 * row-major; bias[l]: device [dims[l+1]]; logits: device [cap_rows[0], dims[n_layers]].
 * n_layers must equal blocks->n_hops.  fp32 storage, fp32 accumulation on the matrix cores. */
int32_t dci_sage_forward(dci_ctx* ctx, const dci_blocks* blocks, const float* x_in, int32_t n_layers,
                         const int32_t* dims, const float* const* w_self, const float* const* w_neigh,
                         const float* const* bias, float* logits);

/* The same forward pass for the other model variants of Table III:
 *   DCI_MODEL_SAGE_MEAN  as dci_sage_forward;
 *   DCI_MODEL_SAGE_SUM   GraphSAGE with the sum aggregator (the table's "Agg: sum"):
 *                        m_i = sum of x[src] over the row's edges;
 *   DCI_MODEL_GCN_AVG    GCN with the averaging aggregator (the table's "Agg: avg"): one weight
 *                        matrix per layer, y_i = a_i w_neigh[l] + bias[l] with a_i the mean over
 *                        node i itself and its sampled neighbours; w_self is ignored (may be NULL).
 * All other arguments as for dci_sage_forward. */
#define DCI_MODEL_SAGE_MEAN 0
#define DCI_MODEL_SAGE_SUM 1
#define DCI_MODEL_GCN_AVG 2
int32_t dci_gnn_forward(dci_ctx* ctx, const dci_blocks* blocks, const float* x_in, int32_t n_layers,
                        const int32_t* dims, int32_t model, const float* const* w_self,
                        const float* const* w_neigh, const float* const* bias, float* logits);

/* Feature gather and forward pass in one call, for the case that the gathered rows are wanted only
 * as the model's input (Section IV, framework paragraph: rows come from GPU memory on a hit, from
 * host memory on a miss; Section V-B: loading features is the stage the feature cache shortens).
 * The logits are those of dci_gather_features(blocks->nodes) followed by dci_gnn_forward, but rows
 * that sit in the feature cache and are needed only as neighbours of the input layer are not copied:
 * the input layer's aggregation reads them where they are.  Copied into x (device
 * [blocks->cap_nodes, F], scratch) are the rows that miss - each crosses the host link once, however
 * many edges use it - and the rows of F_{L-1}, which the input layer's dense product reads as a
 * matrix; the other rows of x are left as they were.  dims[0] must equal graph->feat_dim.  The
 * workspace must hold dci_gather_forward_workspace_bytes(blocks->cap_nodes, blocks->cap_rows,
 * n_layers, dims) bytes.  stats (nullable): DCI_STAT_FEAT_HITS / _MISSES and the byte counters as
 * dci_gather_features would count them (once per input node). */
size_t dci_gather_forward_workspace_bytes(int64_t cap_nodes, const int64_t* cap_rows, int32_t n_layers,
                                          const int32_t* dims);
int32_t dci_gather_forward(dci_ctx* ctx, const dci_graph* graph, const dci_cache* cache,
                           const dci_blocks* blocks, float* x, int32_t n_layers, const int32_t* dims,
                           int32_t model, const float* const* w_self, const float* const* w_neigh,
                           const float* const* bias, float* logits, uint64_t* stats);

/* ---- inference over many batches, several in flight ----------------------------------------- */

/* Inference over the batches [first_batch, first_batch + n_batches) of the seed list (Section V-B: a
 * batch passes through sampling, feature loading and model computation, and the inference time is
 * the sum over all test batches; Fig. 1).  Batch b covers seeds[b*batch_size .. min(n_seeds,
 * (b+1)*batch_size)), uses RNG batch index b and goes, whole, through dci_sample_khop ->
 * dci_gather_features -> dci_gnn_forward on lane (b - first_batch) mod n_lanes; its logits land in
 * rows b*batch_size .. of `logits` (device [n_seeds, dims[n_hops]]).  A lane is a context - its own
 * stream, and a workspace that covers dci_sample_workspace_bytes and dci_sage_workspace_bytes (with
 * DCI_OPT_FUSED_INPUT: dci_gather_forward_workspace_bytes) for these sizes - with its own batch buffers (blocks sized by dci_blocks_bounds for batch_size
 * seeds; x: device [blocks->cap_nodes, F]).  Batches on different lanes run concurrently, so the
 * sampling of one batch overlaps the feature loading and the model computation of others; the
 * graph, the cache, the weights and the seeds are shared and only read; `stats` (nullable) is
 * shared and updated atomically.  The result of every batch is exactly what the three calls give
 * one after the other on one context.  The call only enqueues: results are valid after dci_sync
 * on every lane's context; each lane's blocks / x then hold the last batch that lane ran.  Work
 * already enqueued on a lane's stream is waited for by that stream as usual; the caller must have
 * made the inputs visible to all lanes' streams (e.g. by a device-wide synchronisation after
 * dci_fill_caches).  No two lanes may share a context or a buffer (DCI_ERR_INVALID_ARG); at most
 * DCI_MAX_LANES lanes.  model, dims, weights: as for dci_gnn_forward with n_layers = n_hops. */
#define DCI_MAX_LANES 16
typedef struct {
  dci_ctx* ctx;
  dci_blocks* blocks;
  float* x;
} dci_lane;
int32_t dci_infer_batches(const dci_lane* lanes, int32_t n_lanes, const dci_graph* graph,
                          const dci_cache* cache, const int64_t* seeds, int64_t n_seeds, int32_t batch_size,
                          int64_t first_batch, int64_t n_batches, const int32_t* fanouts, int32_t n_hops,
                          uint64_t rng_seed, int32_t model, const int32_t* dims, const float* const* w_self,
                          const float* const* w_neigh, const float* const* bias, float* logits,
                          uint64_t* stats);

#ifdef __cplusplus
}
#endif
#endif /* DCI_H_ */
