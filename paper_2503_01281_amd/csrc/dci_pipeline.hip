// Inference over consecutive mini-batches with several of them in flight (Section V-B: a batch goes
// through three stages - sampling, feature loading, model computation - and inference time is their
// sum over all test batches; Fig. 1).  The stages of ONE batch depend on each other, those of
// different batches do not: the sampler is a pure function of (seed, batch index), the caches are
// read-only.  So batch b runs, whole, on lane (b - first_batch) mod n_lanes - a lane being a context
// (its own stream and workspace) with its own batch buffers - and the short latency-bound sampling
// kernels of one batch, the bandwidth-bound gather / aggregation of another and the matrix-core
// layers of a third share the chip.  Nothing here waits: the calls enqueue and return.
#include "dci_internal.h"

extern "C" int32_t dci_infer_batches(const dci_lane* lanes, int32_t n_lanes, const dci_graph* graph,
                                     const dci_cache* cache, const int64_t* seeds, int64_t n_seeds,
                                     int32_t batch_size, int64_t first_batch, int64_t n_batches,
                                     const int32_t* fanouts, int32_t n_hops, uint64_t rng_seed, int32_t model,
                                     const int32_t* dims, const float* const* w_self, const float* const* w_neigh,
                                     const float* const* bias, float* logits, uint64_t* stats) {
  if (!lanes || n_lanes < 1 || !lanes[0].ctx) return DCI_ERR_INVALID_ARG;
  dci_ctx* first = lanes[0].ctx;
  if (n_lanes > DCI_MAX_LANES) return dci::fail(first, DCI_ERR_INVALID_ARG, "infer_batches: at most %d lanes", DCI_MAX_LANES);
  for (int32_t k = 0; k < n_lanes; ++k) {
    if (!lanes[k].ctx || !lanes[k].blocks || !lanes[k].x)
      return dci::fail(first, DCI_ERR_INVALID_ARG, "infer_batches: lane %d has a null context, blocks or row buffer", k);
    if (lanes[k].ctx->device != first->device)
      return dci::fail(first, DCI_ERR_INVALID_ARG, "infer_batches: lane %d is on another GPU", k);
    for (int32_t j = 0; j < k; ++j)
      if (lanes[j].ctx == lanes[k].ctx || lanes[j].blocks == lanes[k].blocks || lanes[j].x == lanes[k].x ||
          lanes[j].blocks->nodes == lanes[k].blocks->nodes || lanes[j].blocks->counts == lanes[k].blocks->counts)
        return dci::fail(first, DCI_ERR_INVALID_ARG, "infer_batches: lanes %d and %d share a context or a buffer", j, k);
  }
  if (!graph || !seeds || !fanouts || !dims || !logits || batch_size < 1 || first_batch < 0 || n_batches < 0 || n_seeds < 0)
    return dci::fail(first, DCI_ERR_INVALID_ARG, "infer_batches: null argument or negative size");
  if (n_hops < 1 || n_hops > DCI_MAX_HOPS) return dci::fail(first, DCI_ERR_INVALID_ARG, "infer_batches: n_hops must be 1..%d", DCI_MAX_HOPS);
  const int64_t width = dims[n_hops];
  for (int64_t k = 0; k < n_batches; ++k) {
    const int64_t b = first_batch + k;
    const int64_t lo = b * (int64_t)batch_size;
    if (lo >= n_seeds) break;
    const int64_t n = lo + batch_size < n_seeds ? batch_size : n_seeds - lo;
    const dci_lane& lane = lanes[k % n_lanes];
    dci_ctx* ctx = lane.ctx;
    int32_t rc = dci_sample_khop(ctx, graph, cache, seeds + lo, n, (uint64_t)b, fanouts, n_hops, rng_seed, lane.blocks, stats);
    if (rc == DCI_OK && ctx->fused_input) {
      rc = dci_gather_forward(ctx, graph, cache, lane.blocks, lane.x, n_hops, dims, model, w_self, w_neigh, bias,
                              logits + lo * width, stats);
    } else {
      if (rc == DCI_OK)
        rc = dci_gather_features(ctx, graph, cache, lane.blocks->nodes, lane.blocks->cap_nodes,
                                 lane.blocks->counts + n_hops, lane.x, stats);
      if (rc == DCI_OK)
        rc = dci_gnn_forward(ctx, lane.blocks, lane.x, n_hops, dims, model, w_self, w_neigh, bias, logits + lo * width);
    }
    if (rc != DCI_OK) {
      if (ctx != first) dci::fail(first, rc, "infer_batches: batch %lld on lane %d: %s", (long long)b, (int)(k % n_lanes), ctx->err);
      return rc;
    }
  }
  return DCI_OK;
}
