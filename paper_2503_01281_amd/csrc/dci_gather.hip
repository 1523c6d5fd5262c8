// Cache-aware feature gather (Section IV, framework paragraph; Section IV-B, first paragraph):
// a row comes from the HBM feature cache when feat_remap[id] >= 0 and from the host feature
// matrix (zero-copy over the host link) otherwise.
//
// The copy is bandwidth bound.  A row is handled by a group of lanes (a whole wavefront for
// rows of 64 or more 16-byte chunks, a fraction for narrow rows); consecutive lanes move
// consecutive 16-byte chunks, up to four loads in flight per lane before the first store, and the
// id / remap lookups of the next two rows are issued while the current row is copied.  Rows need
// only 4-byte alignment: gfx950 global memory takes under-aligned 16-byte accesses, and the
// F % 4 trailing floats are moved one per lane.
#include "dci_internal.h"

namespace dci {

constexpr int kGatherBlock = 256;
constexpr int kGatherBlocksPerCu = 16;

typedef float4 __attribute__((aligned(4))) float4_u;  // 16-byte access at 4-byte alignment
typedef float2 __attribute__((aligned(4))) float2_u;

template <int V>
struct GVec;
template <>
struct GVec<4> { typedef float4 reg; typedef float4_u mem; };
template <>
struct GVec<2> { typedef float2 reg; typedef float2_u mem; };
template <>
struct GVec<1> { typedef float reg; typedef float mem; };

struct GatherCounts {
  unsigned long long hits = 0, misses = 0, copied = 0;
};

// Copies rows [0, n) of the id list: a group of 2^lpr_log2 lanes per row, workgroup `block` of `n_blocks`
// taking every n_blocks-th slice of rows.  rowref (nullable) receives every row's cache slot or -1.
template <int V>
__device__ __forceinline__ void copy_rows(const long long* __restrict__ ids, long long n,
                                          const int* __restrict__ remap, const float* __restrict__ cache,
                                          const float* __restrict__ feat, int F, int lpr_log2,
                                          float* __restrict__ out, int* __restrict__ rowref, int block, int n_blocks,
                                          GatherCounts& cnt) {
  typedef typename GVec<V>::reg reg_t;
  typedef typename GVec<V>::mem mem_t;
  const int chunks = F / V, tail = F % V;
  const int lpr = 1 << lpr_log2;  // lanes per row
  const int rows_per_block = kGatherBlock >> lpr_log2;
  const int sub = (int)threadIdx.x >> lpr_log2;  // row within the block's slice
  const int cl = (int)threadIdx.x & (lpr - 1);   // first chunk of this lane
  const long long stride = (long long)n_blocks * rows_per_block;

  long long i = (long long)block * rows_per_block + sub;
  long long id = i < n ? ids[i] : 0;
  int r = (i < n && remap) ? remap[id] : -1;
  long long i2 = i + stride;
  long long id2 = i2 < n ? ids[i2] : 0;
  while (i < n) {
    // look-ups of the following rows go out before this row's copy
    const int r2 = (i2 < n && remap) ? remap[id2] : -1;
    const long long i3 = i2 + stride;
    const long long id3 = i3 < n ? ids[i3] : 0;

    const float* src = r >= 0 ? cache + (long long)r * F : feat + id * F;
    float* dst = out + i * F;
    if (cl == 0) {
      if (r >= 0) ++cnt.hits; else ++cnt.misses;
      ++cnt.copied;
      if (rowref) rowref[i] = r;
    }
    for (int c0 = cl; c0 < chunks; c0 += 4 * lpr) {
      reg_t v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (c0 + u * lpr < chunks) v[u] = reinterpret_cast<const mem_t*>(src)[c0 + u * lpr];
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (c0 + u * lpr < chunks) reinterpret_cast<mem_t*>(dst)[c0 + u * lpr] = v[u];
    }
    if (cl < tail) dst[V * chunks + cl] = src[V * chunks + cl];

    i = i2; id = id2; r = r2;
    i2 = i3; id2 = id3;
  }
}

// Hit / miss / copied totals leave a gather kernel as one triple per workgroup and are folded by a second,
// tiny kernel: thousands of atomics on one counter serialise in L2 for longer than the copy takes
// (measured: +30 us for 4096 workgroups).
__device__ __forceinline__ void store_partials(GatherCounts cnt, unsigned long long* __restrict__ partials) {
  __shared__ unsigned long long s_h[kGatherBlock / kWave], s_m[kGatherBlock / kWave], s_c[kGatherBlock / kWave];
  const unsigned long long hits = wave_sum_u64(cnt.hits), misses = wave_sum_u64(cnt.misses), copied = wave_sum_u64(cnt.copied);
  if (lane_id() == 0) {
    s_h[threadIdx.x / kWave] = hits;
    s_m[threadIdx.x / kWave] = misses;
    s_c[threadIdx.x / kWave] = copied;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    unsigned long long h = 0, m = 0, c = 0;
    for (int w = 0; w < kGatherBlock / kWave; ++w) {
      h += s_h[w];
      m += s_m[w];
      c += s_c[w];
    }
    partials[3 * blockIdx.x] = h;
    partials[3 * blockIdx.x + 1] = m;
    partials[3 * blockIdx.x + 2] = c;
  }
}

template <int V>
__global__ __launch_bounds__(kGatherBlock) void k_gather(const long long* __restrict__ ids, long long n_max,
                                                         const long long* __restrict__ n_dev,
                                                         const int* __restrict__ remap,
                                                         const float* __restrict__ cache,
                                                         const float* __restrict__ feat, int F, int lpr_log2,
                                                         float* __restrict__ out,
                                                         unsigned long long* __restrict__ partials) {
  long long n = n_dev ? *n_dev : n_max;
  if (n > n_max) n = n_max;
  GatherCounts cnt;
  copy_rows<V>(ids, n, remap, cache, feat, F, lpr_log2, out, nullptr, (int)blockIdx.x, (int)gridDim.x, cnt);
  if (partials) store_partials(cnt, partials);
}

// The selective gather of dci_gather_forward: every row's cache slot (or -1) is noted in rowref[i]; the
// row itself is copied only if it lies below *n_dense_dev (the rows of F_{L-1}, which the dense layer reads
// as a matrix) or misses (so that it crosses the host link once, not once per edge that uses it).
// Some workgroups copy the rows of F_{L-1} like the plain gather; the others (interleaved with them, so
// that the two kinds of work run side by side instead of one after the other; the shares follow the bytes
// each kind moves for this batch's sizes) go over the
// rest with one lane per row - 64 dependent id -> remap chains in flight per wavefront instead of one per
// lane group, because most of these rows are only looked up - and the rows among them that missed are then
// listed in LDS and copied a lane group per row, two rows per group in flight.
template <int V>
__global__ __launch_bounds__(kGatherBlock) void k_gather_select(const long long* __restrict__ ids, long long n_max,
                                                                const long long* __restrict__ n_dev,
                                                                const int* __restrict__ remap,
                                                                const float* __restrict__ cache,
                                                                const float* __restrict__ feat, int F, int lpr_log2,
                                                                float* __restrict__ out,
                                                                unsigned long long* __restrict__ partials,
                                                                int* __restrict__ rowref,
                                                                const long long* __restrict__ n_dense_dev) {
  typedef typename GVec<V>::reg reg_t;
  typedef typename GVec<V>::mem mem_t;
  long long n = *n_dev;
  if (n > n_max) n = n_max;
  long long n_dense = *n_dense_dev;
  if (n_dense > n) n_dense = n;
  GatherCounts cnt;
  // Workgroup b copies dense rows iff floor((b+1) nd / G) != floor(b nd / G): nd of the G workgroups, evenly
  // spread.  nd follows the work: 8F bytes per dense row - but no less than 2 KB, since narrow rows are bound by
  // the latency of their id -> slot -> row chain, not by their bytes - against about 160 bytes per looked-up row
  // (id, a sector of the remap, the slot note).
  const long long G = (long long)gridDim.x, b = (long long)blockIdx.x;
  long long nd;
  {
    const double dense_bytes = (double)n_dense * (8.0 * F > 2048.0 ? 8.0 * F : 2048.0), look_bytes = (double)(n - n_dense) * 160.0;
    nd = (long long)((double)G * dense_bytes / (dense_bytes + look_bytes + 1.0) + 0.5);
    if (nd < 1) nd = 1;
    if (nd > G - 1) nd = G - 1;
  }
  const long long before = b * nd / G;  // dense workgroups among 0 .. b-1
  if ((b + 1) * nd / G != before) {
    copy_rows<V>(ids, n_dense, remap, cache, feat, F, lpr_log2, out, rowref, (int)before, (int)nd, cnt);
  } else {
    const long long q = b - before, n_look = G - nd;  // this workgroup's index among the look-up ones, and their number
    // 256 rows per round: every lane looks one row up; the rows that missed are listed in LDS and then copied
    // like the dense ones, a lane group per row, so that narrow rows keep all lanes busy.
    __shared__ int s_list[kGatherBlock];
    __shared__ int s_count;
    const int chunks = F / V, tail = F % V;
    const int lpr = 1 << lpr_log2;
    const int rows_per_round = kGatherBlock >> lpr_log2;
    const int sub = (int)threadIdx.x >> lpr_log2, cl = (int)threadIdx.x & (lpr - 1);
    for (long long base = n_dense + q * kGatherBlock; base < n; base += n_look * kGatherBlock) {
      if (threadIdx.x == 0) s_count = 0;
      __syncthreads();
      const long long i = base + threadIdx.x;
      const bool valid = i < n;
      const long long id = valid ? ids[i] : 0;
      const int r = (valid && remap) ? remap[id] : -1;
      if (valid) {
        rowref[i] = r;
        if (r >= 0) ++cnt.hits; else ++cnt.misses;
      }
      if (valid && r < 0) {
        ++cnt.copied;
        s_list[atomicAdd(&s_count, 1)] = (int)threadIdx.x;  // the order within the list does not matter
      }
      __syncthreads();
      const int n_miss = s_count;
      for (int k0 = sub; k0 < n_miss; k0 += 2 * rows_per_round) {
        // two rows per lane group in flight
        const int k1 = k0 + rows_per_round;
        const long long ia = base + s_list[k0], ib = k1 < n_miss ? base + s_list[k1] : ia;
        const float* sa = feat + ids[ia] * F;
        const float* sb = feat + ids[ib] * F;
        float* da = out + ia * F;
        float* db = out + ib * F;
        for (int c0 = cl; c0 < chunks; c0 += lpr) {
          const reg_t va = reinterpret_cast<const mem_t*>(sa)[c0];
          const reg_t vb = reinterpret_cast<const mem_t*>(sb)[c0];
          reinterpret_cast<mem_t*>(da)[c0] = va;
          if (k1 < n_miss) reinterpret_cast<mem_t*>(db)[c0] = vb;
        }
        if (cl < tail) {
          const float ta = sa[V * chunks + cl], tb = sb[V * chunks + cl];
          da[V * chunks + cl] = ta;
          if (k1 < n_miss) db[V * chunks + cl] = tb;
        }
      }
      __syncthreads();  // the list is rewritten in the next round
    }
  }
  if (partials) store_partials(cnt, partials);
}

__global__ __launch_bounds__(kGatherBlock) void k_fold_gather_stats(const unsigned long long* __restrict__ partials,
                                                                    int n_blocks, unsigned long long row_bytes,
                                                                    unsigned long long* stats) {
  unsigned long long h = 0, m = 0, c = 0;
  for (int b = (int)threadIdx.x; b < n_blocks; b += kGatherBlock) {
    h += partials[3 * b];
    m += partials[3 * b + 1];
    c += partials[3 * b + 2];
  }
  __shared__ unsigned long long s_h[kGatherBlock / kWave], s_m[kGatherBlock / kWave], s_c[kGatherBlock / kWave];
  h = wave_sum_u64(h);
  m = wave_sum_u64(m);
  c = wave_sum_u64(c);
  if (lane_id() == 0) {
    s_h[threadIdx.x / kWave] = h;
    s_m[threadIdx.x / kWave] = m;
    s_c[threadIdx.x / kWave] = c;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    h = m = c = 0;
    for (int w = 0; w < kGatherBlock / kWave; ++w) {
      h += s_h[w];
      m += s_m[w];
      c += s_c[w];
    }
    if (c) atomicAdd(&stats[DCI_STAT_ROWS_COPIED], c);
    atomicAdd(&stats[DCI_STAT_FEAT_HITS], h);
    atomicAdd(&stats[DCI_STAT_FEAT_MISSES], m);
    // a gathered row is read once, from the tier that holds it
    if (h) atomicAdd(&stats[DCI_STAT_BYTES_HBM], h * row_bytes);
    if (m) atomicAdd(&stats[DCI_STAT_BYTES_HOST], m * row_bytes);
  }
}

size_t gather_partials_bytes(const dci_ctx* ctx) {
  return (size_t)ctx->num_cus * kGatherBlocksPerCu * 3 * sizeof(unsigned long long);
}

int32_t gather_launch(dci_ctx* ctx, const dci_graph* g, const dci_cache* cache, const int64_t* ids, int64_t n_max,
                      const int64_t* n_dev, float* out, uint64_t* stats, void* partials_buf, int32_t* rowref,
                      const int64_t* n_dense_dev, int64_t n_dense_max) {
  const int F = g->feat_dim;
  const float* fcache = cache ? cache->feat_cache : nullptr;
  const int* remap = cache ? cache->feat_remap : nullptr;
  // 16-byte chunks when rows start 16-byte aligned; otherwise 8-byte chunks (under-aligned 16-byte
  // accesses work but measured slower than aligned 8-byte ones)
  auto aligned = [](const void* p, size_t a) { return p == nullptr || (reinterpret_cast<uintptr_t>(p) % a) == 0; };
  int V = 1;
  if (F % 4 == 0 && aligned(g->feat, 16) && aligned(out, 16) && aligned(fcache, 16)) V = 4;
  else if (F % 2 == 0 && aligned(g->feat, 8) && aligned(out, 8) && aligned(fcache, 8)) V = 2;
  const int chunks = F / V;
  int lpr_log2 = 0;
  while ((1 << lpr_log2) < chunks && lpr_log2 < 6) ++lpr_log2;
  const int rows_per_block = kGatherBlock >> lpr_log2;
  const int64_t cap = (int64_t)ctx->num_cus * kGatherBlocksPerCu;
  auto blocks_for = [&](int64_t rows, int per_block) {
    int64_t b = (rows + per_block - 1) / per_block;
    if (b > cap) b = cap;
    return b < 1 ? (int64_t)1 : b;
  };
  int64_t blocks = blocks_for(n_max, rows_per_block);
  {
    Timed timed(ctx, DCI_K_GATHER);
    const long long* ids_ = reinterpret_cast<const long long*>(ids);
    const long long* nd_ = reinterpret_cast<const long long*>(n_dev);
    const long long* dn_ = reinterpret_cast<const long long*>(n_dense_dev);
    unsigned long long* st = stats ? reinterpret_cast<unsigned long long*>(partials_buf) : nullptr;
    if (rowref) {
      if (!n_dev || !n_dense_dev) return fail(ctx, DCI_ERR_INVALID_ARG, "selective gather needs device-side row counts");
      // workgroups for both kinds of work; the kernel shares them out from the batch's own sizes (both parts
      // walk their rows with a grid stride, so any split is correct)
      blocks = blocks_for(n_dense_max, rows_per_block) + blocks_for(n_max, kGatherBlock);
      if (blocks > cap) blocks = cap;
      if (blocks < 2) blocks = 2;
      if (V == 4)
        hipLaunchKernelGGL((k_gather_select<4>), dim3((int)blocks), dim3(kGatherBlock), 0, ctx->stream, ids_,
                           (long long)n_max, nd_, remap, fcache, g->feat, F, lpr_log2, out, st, rowref, dn_);
      else if (V == 2)
        hipLaunchKernelGGL((k_gather_select<2>), dim3((int)blocks), dim3(kGatherBlock), 0, ctx->stream, ids_,
                           (long long)n_max, nd_, remap, fcache, g->feat, F, lpr_log2, out, st, rowref, dn_);
      else
        hipLaunchKernelGGL((k_gather_select<1>), dim3((int)blocks), dim3(kGatherBlock), 0, ctx->stream, ids_,
                           (long long)n_max, nd_, remap, fcache, g->feat, F, lpr_log2, out, st, rowref, dn_);
    } else if (V == 4)
      hipLaunchKernelGGL((k_gather<4>), dim3((int)blocks), dim3(kGatherBlock), 0, ctx->stream, ids_, (long long)n_max,
                         nd_, remap, fcache, g->feat, F, lpr_log2, out, st);
    else if (V == 2)
      hipLaunchKernelGGL((k_gather<2>), dim3((int)blocks), dim3(kGatherBlock), 0, ctx->stream, ids_, (long long)n_max,
                         nd_, remap, fcache, g->feat, F, lpr_log2, out, st);
    else
      hipLaunchKernelGGL((k_gather<1>), dim3((int)blocks), dim3(kGatherBlock), 0, ctx->stream, ids_, (long long)n_max,
                         nd_, remap, fcache, g->feat, F, lpr_log2, out, st);
  }
  DCI_LAUNCH_CHECK(ctx);
  if (stats) {
    hipLaunchKernelGGL(k_fold_gather_stats, dim3(1), dim3(kGatherBlock), 0, ctx->stream,
                       reinterpret_cast<const unsigned long long*>(partials_buf), (int)blocks,
                       (unsigned long long)F * 4ull, reinterpret_cast<unsigned long long*>(stats));
    DCI_LAUNCH_CHECK(ctx);
  }
  return DCI_OK;
}

}  // namespace dci

extern "C" int32_t dci_gather_features(dci_ctx* ctx, const dci_graph* graph, const dci_cache* cache,
                                       const int64_t* node_ids, int64_t n_max, const int64_t* n_dev, float* out,
                                       uint64_t* stats) {
  if (!ctx) return DCI_ERR_INVALID_ARG;
  if (!graph || !graph->feat || graph->feat_dim < 1 || graph->num_nodes < 1)
    return dci::fail(ctx, DCI_ERR_INVALID_ARG, "graph: feature matrix missing or feat_dim < 1");
  if (n_max < 0 || (n_max > 0 && (!node_ids || !out)))
    return dci::fail(ctx, DCI_ERR_INVALID_ARG, "node_ids / out: null or negative count");
  if (cache && (!cache->feat_remap || (cache->feat_rows > 0 && !cache->feat_cache)))
    return dci::fail(ctx, DCI_ERR_INVALID_ARG, "cache: null feature arrays");
  if ((reinterpret_cast<uintptr_t>(graph->feat) | reinterpret_cast<uintptr_t>(out) |
       (cache ? reinterpret_cast<uintptr_t>(cache->feat_cache) : 0)) & 3)
    return dci::fail(ctx, DCI_ERR_INVALID_ARG, "feature arrays must be 4-byte aligned");
  if (n_max == 0) return DCI_OK;
  void* partials = nullptr;
  if (stats) {
    dci::Arena ar(ctx->ws, ctx->ws_bytes);
    partials = ar.take<char>(dci::gather_partials_bytes(ctx));
    if (!ar.ok())
      return dci::fail(ctx, DCI_ERR_CAPACITY, "workspace holds %zu bytes, gather statistics need %zu", ctx->ws_bytes,
                       ar.off);
  }
  return dci::gather_launch(ctx, graph, cache, node_ids, n_max, n_dev, out, stats, partials, nullptr, nullptr, 0);
}
