// CPU oracle for the dual-cache GNN inference path (DCI, arXiv 2503.01281).
//
// TEST INFRASTRUCTURE ONLY.  This is a plain, sequential, deliberately slow statement of
// what the path computes.  It shares no code with the GPU library and must never be
// called from the product path: only the tests, the smoke check and the benchmark's
// "cpu_baseline" leg load it.  Host pointers everywhere.
//
// What each part follows:
//   * sampling / mini-batch blocks ... Section II-C (neighbour sampling with a fan-out per
//     hop; the in-neighbours of a target are one CSC column) and Section IV (a cache only
//     changes where bytes are read from, never which bytes);
//   * counting ..................... Section IV-B, first paragraph (visits per node, and
//     accesses per adjacency element, recorded while pre-sampling);
//   * capacity split ............... Eq. (1);
//   * feature-cache fill ........... Section IV-B, first paragraph ("greater than the
//     average" first, the rest afterwards, no sort);
//   * adjacency-cache fill ......... Algorithm 1 and Fig. 6: node-granular reading (oracle_fill_adj) and the
//     element-granular form as printed (oracle_fill_adj_element);
//   * feature gather ............... Section IV, framework paragraph (hit: GPU memory,
//     miss: host memory; same row either way);
//   * model ........................ GraphSAGE with mean aggregation (Table III family), plus the
//     table's own variants: GraphSAGE with the sum aggregator and GCN with the averaging one.
//
// The random numbers of the sampler come from Philox4x32-10 (Salmon et al., SC'11) used
// as a counter-based generator keyed by (seed; node, batch, hop, slot), so a sample is a
// pure function of those five values and independent of execution order.
//
// Pins: every function below is pinned by tests/test_oracle_*.py (known-answer vectors,
// brute force, closed forms, invariants).  Nothing here is "parity unpinned" except the
// numeric hit rates, for which the paper prints no table.

#include <algorithm>
#include <chrono>
#include <cstdint>
#include <cstring>
#include <numeric>
#include <thread>
#include <unordered_map>
#include <vector>

typedef unsigned __int128 u128;

// ---------------------------------------------------------------------------------------
// Philox4x32-10.  Round: (c0,c1,c2,c3) -> (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1,
// lo(M0*c0)); the key is bumped by the two Weyl constants between rounds.
static void philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  const uint64_t M0 = 0xD2511F53ull, M1 = 0xCD9E8D57ull;
  const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    uint64_t p0 = M0 * (uint64_t)c0;
    uint64_t p1 = M1 * (uint64_t)c2;
    uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    uint32_t n1 = (uint32_t)p1;
    uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += W0; k1 += W1;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Uniform integer in [0, m): the high 64 bits of (64 random bits) * m.
// key = (seed lo, seed hi); counter = (node lo, node hi, batch, hop<<24 | slot).
static uint64_t uniform_below(uint64_t rng_seed, int64_t node, uint64_t batch_index, int32_t hop,
                              int32_t slot, uint64_t m) {
  uint32_t key[2] = {(uint32_t)rng_seed, (uint32_t)(rng_seed >> 32)};
  uint32_t ctr[4] = {(uint32_t)(uint64_t)node, (uint32_t)((uint64_t)node >> 32), (uint32_t)batch_index,
                     ((uint32_t)hop << 24) | (uint32_t)slot};
  uint32_t x[4];
  philox4x32_10(ctr, key, x);
  uint64_t u = (uint64_t)x[0] | ((uint64_t)x[1] << 32);
  return (uint64_t)(((u128)u * (u128)m) >> 64);
}

// Positions (offsets into the node's neighbour list) chosen for one frontier node:
// all of them, in list order, when deg <= fanout; otherwise a uniform fanout-subset
// without replacement by Floyd's algorithm, reported in the order the algorithm appends.
static int32_t sample_positions(uint64_t rng_seed, uint64_t batch_index, int32_t hop, int64_t node,
                                int64_t deg, int32_t fanout, int64_t* pos) {
  if (deg <= fanout) {
    for (int64_t p = 0; p < deg; ++p) pos[p] = p;
    return (int32_t)deg;
  }
  for (int32_t slot = 0; slot < fanout; ++slot) {
    int64_t j = deg - fanout + slot;
    int64_t t = (int64_t)uniform_below(rng_seed, node, batch_index, hop, slot, (uint64_t)(j + 1));
    bool seen = false;
    for (int32_t q = 0; q < slot; ++q) seen = seen || (pos[q] == t);
    pos[slot] = seen ? j : t;
  }
  return fanout;
}

// One mini-batch: frontiers F_0 (the seeds) .. F_L and one bipartite block per hop.
struct Batch {
  std::vector<int64_t> nodes;                     // F_L; F_h is its prefix of length n_nodes[h]
  std::vector<int64_t> n_nodes;                   // L+1
  std::vector<std::vector<int64_t>> blk_indptr;   // per hop, n_nodes[h]+1
  std::vector<std::vector<int32_t>> blk_src;      // per hop, local ids into F_{h+1}
  std::vector<std::vector<int64_t>> src_global;   // per hop, global ids of the sampled neighbours
  std::vector<std::vector<int64_t>> src_pos;      // per hop, position of each sample in its list
};

static void sample_batch(const int64_t* indptr, const int64_t* indices, const int64_t* seeds, int64_t n_seeds,
                         uint64_t batch_index, const int32_t* fanouts, int32_t n_hops, uint64_t rng_seed,
                         Batch* out) {
  Batch& b = *out;
  b.nodes.assign(seeds, seeds + n_seeds);
  b.n_nodes.assign(1, n_seeds);
  b.blk_indptr.assign(n_hops, {});
  b.blk_src.assign(n_hops, {});
  b.src_global.assign(n_hops, {});
  b.src_pos.assign(n_hops, {});
  std::unordered_map<int64_t, int32_t> local;  // global id -> index in F
  for (int64_t i = 0; i < n_seeds; ++i) local.emplace(seeds[i], (int32_t)i);
  std::vector<int64_t> pos;
  for (int32_t h = 0; h < n_hops; ++h) {
    const int32_t f = fanouts[h];
    const int64_t n_h = b.n_nodes[h];
    pos.resize((size_t)std::max(f, 1));
    b.blk_indptr[h].assign(1, 0);
    for (int64_t i = 0; i < n_h; ++i) {
      const int64_t v = b.nodes[i];
      const int64_t start = indptr[v], deg = indptr[v + 1] - indptr[v];
      const int32_t c = sample_positions(rng_seed, batch_index, h, v, deg, f, pos.data());
      for (int32_t s = 0; s < c; ++s) {
        const int64_t u = indices[start + pos[s]];
        auto it = local.find(u);
        if (it == local.end()) {  // first appearance: next free local id, appended to F
          it = local.emplace(u, (int32_t)b.nodes.size()).first;
          b.nodes.push_back(u);
        }
        b.blk_src[h].push_back(it->second);
        b.src_global[h].push_back(u);
        b.src_pos[h].push_back(pos[s]);
      }
      b.blk_indptr[h].push_back((int64_t)b.blk_src[h].size());
    }
    b.n_nodes.push_back((int64_t)b.nodes.size());
  }
}

extern "C" {

void oracle_philox4x32_10(const uint32_t* ctr, const uint32_t* key, uint32_t* out) {
  philox4x32_10(ctr, key, out);
}

uint64_t oracle_uniform_below(uint64_t rng_seed, int64_t node, uint64_t batch_index, int32_t hop,
                              int32_t slot, uint64_t m) {
  return uniform_below(rng_seed, node, batch_index, hop, slot, m);
}

int32_t oracle_sample_positions(uint64_t rng_seed, uint64_t batch_index, int32_t hop, int64_t node,
                                int64_t deg, int32_t fanout, int64_t* pos) {
  return sample_positions(rng_seed, batch_index, hop, node, deg, fanout, pos);
}

// Samples one mini-batch.  Buffers are caller-allocated:
//   nodes[cap_nodes], n_nodes[n_hops+1], n_edges[n_hops],
//   blk_indptr[h] -> int64[n_nodes[h]+1], blk_src[h] -> int32[cap_edges[h]],
//   src_global[h], src_pos[h] -> int64[cap_edges[h]] (each nullable).
// Returns 0, or -2 when a capacity is too small (n_nodes / n_edges then hold what is needed).
int32_t oracle_sample_khop(const int64_t* indptr, const int64_t* indices, const int64_t* seeds,
                           int64_t n_seeds, uint64_t batch_index, const int32_t* fanouts, int32_t n_hops,
                           uint64_t rng_seed, int64_t* nodes, int64_t cap_nodes, int64_t* n_nodes,
                           int64_t* n_edges, int64_t** blk_indptr, int32_t** blk_src, int64_t** src_global,
                           int64_t** src_pos, const int64_t* cap_edges) {
  Batch b;
  sample_batch(indptr, indices, seeds, n_seeds, batch_index, fanouts, n_hops, rng_seed, &b);
  int32_t rc = 0;
  for (int32_t h = 0; h <= n_hops; ++h) n_nodes[h] = b.n_nodes[h];
  for (int32_t h = 0; h < n_hops; ++h) {
    n_edges[h] = (int64_t)b.blk_src[h].size();
    if (n_edges[h] > cap_edges[h]) rc = -2;
  }
  if ((int64_t)b.nodes.size() > cap_nodes) rc = -2;
  if (rc) return rc;
  std::copy(b.nodes.begin(), b.nodes.end(), nodes);
  for (int32_t h = 0; h < n_hops; ++h) {
    std::copy(b.blk_indptr[h].begin(), b.blk_indptr[h].end(), blk_indptr[h]);
    std::copy(b.blk_src[h].begin(), b.blk_src[h].end(), blk_src[h]);
    if (src_global && src_global[h]) std::copy(b.src_global[h].begin(), b.src_global[h].end(), src_global[h]);
    if (src_pos && src_pos[h]) std::copy(b.src_pos[h].begin(), b.src_pos[h].end(), src_pos[h]);
  }
  return 0;
}

// Pre-sampling statistics over the batches [first_batch, first_batch + n_batches) of the
// seed list (batch b covers seeds[b*batch_size .. min(n_seeds,(b+1)*batch_size)) and uses
// RNG batch index rng_batch0 + b):
//   every sampled (node v, list position p): edge_count[indptr[v]+p] += 1, adj_count[v] += 1;
//   every node of the batch's input list F_L: feat_count[u] += 1.
// Counters are accumulated into (not cleared).  edge_count may be NULL.
// totals (nullable): [0] += sampled edges, [1] += input nodes.
int32_t oracle_presample_count(const int64_t* indptr, const int64_t* indices, const int64_t* seeds,
                               int64_t n_seeds, int32_t batch_size, int64_t first_batch, int64_t n_batches,
                               uint64_t rng_batch0, const int32_t* fanouts, int32_t n_hops, uint64_t rng_seed,
                               uint32_t* feat_count, uint32_t* adj_count, uint32_t* edge_count,
                               int64_t* totals) {
  for (int64_t k = 0; k < n_batches; ++k) {
    const int64_t bidx = first_batch + k;
    const int64_t lo = bidx * batch_size;
    if (lo >= n_seeds) break;
    const int64_t hi = std::min<int64_t>(n_seeds, lo + batch_size);
    Batch b;
    sample_batch(indptr, indices, seeds + lo, hi - lo, rng_batch0 + (uint64_t)k, fanouts, n_hops, rng_seed, &b);
    for (int32_t h = 0; h < n_hops; ++h) {
      for (int64_t i = 0; i < b.n_nodes[h]; ++i) {
        const int64_t v = b.nodes[i];
        for (int64_t e = b.blk_indptr[h][i]; e < b.blk_indptr[h][i + 1]; ++e) {
          adj_count[v] += 1;
          if (edge_count) edge_count[indptr[v] + b.src_pos[h][e]] += 1;
        }
      }
      if (totals) totals[0] += (int64_t)b.blk_src[h].size();
    }
    for (int64_t u : b.nodes) feat_count[u] += 1;
    if (totals) totals[1] += (int64_t)b.nodes.size();
  }
  return 0;
}

// Eq. (1) in integers, followed (when spill != 0) by the spill-over rule: a share that exceeds
// what its side can use (the whole adjacency structure, or the whole feature matrix) hands the
// excess to the other side, so that a budget covering the whole dataset caches all of it.
// spill == 0 keeps the shares of Eq. (1) as they are (with t_sample = 0 this is the single-cache
// system the paper compares with in Section V-B: no adjacency cache at all).
void oracle_split(uint64_t C, uint64_t t_sample, uint64_t t_feature, int64_t N, int64_t E, int32_t F,
                  int32_t spill, uint64_t* C_adj, uint64_t* C_feat) {
  const uint64_t tsum = t_sample + t_feature;
  uint64_t adj0 = tsum == 0 ? C / 2 : (uint64_t)(((u128)C * (u128)t_sample) / (u128)tsum);
  uint64_t feat0 = C - adj0;
  const uint64_t A = (uint64_t)(N + 1 + E) * 8ull;
  const uint64_t Ft = (uint64_t)N * (uint64_t)F * 4ull;
  if (!spill) {
  } else if (A <= adj0) {
    adj0 = A;
    feat0 = C - A;
  } else if (Ft <= feat0) {
    feat0 = Ft;
    adj0 = C - Ft;
  }
  *C_adj = adj0;
  *C_feat = feat0;
}

// Feature-cache fill.  k = min(N, C_feat / (4F)) rows.
// policy 0 (the paper's rule): nodes whose visit count exceeds the mean over all N nodes,
//   in ascending id, then the remaining nodes in ascending id; the first k are cached.
// policy 1 (top-k): nodes by visit count descending, ties by ascending id; first k.
// feat_remap[v] = slot or -1; feat_cache[slot,:] = feat[v,:] (feat_cache / feat nullable
// together to compute the remap only).  Returns k.
int64_t oracle_fill_feat(int64_t N, int32_t F, const uint32_t* feat_count, const float* feat,
                         uint64_t C_feat, int32_t policy, int32_t* feat_remap, float* feat_cache) {
  int64_t k = (int64_t)std::min<uint64_t>((uint64_t)N, C_feat / (4ull * (uint64_t)F));
  std::vector<int64_t> order;
  order.reserve((size_t)N);
  if (policy == 0) {
    u128 total = 0;
    for (int64_t v = 0; v < N; ++v) total += feat_count[v];
    for (int64_t v = 0; v < N; ++v)
      if ((u128)feat_count[v] * (u128)N > total) order.push_back(v);
    for (int64_t v = 0; v < N; ++v)
      if (!((u128)feat_count[v] * (u128)N > total)) order.push_back(v);
  } else {
    for (int64_t v = 0; v < N; ++v) order.push_back(v);
    std::stable_sort(order.begin(), order.end(),
                     [&](int64_t x, int64_t y) { return feat_count[x] > feat_count[y]; });
  }
  for (int64_t v = 0; v < N; ++v) feat_remap[v] = -1;
  for (int64_t s = 0; s < k; ++s) {
    const int64_t v = order[(size_t)s];
    feat_remap[v] = (int32_t)s;
    if (feat_cache && feat) std::memcpy(feat_cache + s * F, feat + v * F, sizeof(float) * (size_t)F);
  }
  return k;
}

// Adjacency-cache fill (Algorithm 1, node-granular).  Volume of the whole structure is
// (N+1+E)*8 bytes; if it fits in C_adj everything is cached verbatim (slot = node id).
// Otherwise nodes are ordered by total access count descending (ties: ascending id), and
// the longest prefix whose compacted CSR, 8*(K+1) + 8*sum(deg) bytes, fits is cached:
// lists are concatenated in that order, each in its original element order.
// Outputs: adj_remap[N] (slot or -1), c_indptr[K+1], c_indices[M] (both nullable to compute
// sizes / the remap only), *K_out, *M_out.  cap_K / cap_M guard the output arrays
// (return -2 and set K/M when too small).
int32_t oracle_fill_adj(int64_t N, const int64_t* indptr, const int64_t* indices, const uint32_t* adj_count,
                        uint64_t C_adj, int32_t* adj_remap, int64_t* c_indptr, int64_t cap_K,
                        int64_t* c_indices, int64_t cap_M, int64_t* K_out, int64_t* M_out) {
  const int64_t E = indptr[N];
  const uint64_t volume = (uint64_t)(N + 1 + E) * 8ull;
  std::vector<int64_t> order((size_t)N);
  std::iota(order.begin(), order.end(), (int64_t)0);
  int64_t K = 0, M = 0;
  if (volume <= C_adj) {
    K = N;
    M = E;
  } else {
    std::stable_sort(order.begin(), order.end(),
                     [&](int64_t x, int64_t y) { return adj_count[x] > adj_count[y]; });
    uint64_t used = 8;  // the leading c_indptr entry
    while (K < N) {
      const int64_t v = order[(size_t)K];
      const uint64_t cost = 8ull * (uint64_t)(indptr[v + 1] - indptr[v]) + 8ull;
      if (used + cost > C_adj) break;  // slicing stops at the first node that does not fit
      used += cost;
      M += indptr[v + 1] - indptr[v];
      ++K;
    }
    if (C_adj < 8) K = 0;
  }
  *K_out = K;
  *M_out = M;
  for (int64_t v = 0; v < N; ++v) adj_remap[v] = -1;
  for (int64_t s = 0; s < K; ++s) adj_remap[order[(size_t)s]] = (int32_t)s;
  if (!c_indptr || !c_indices) return 0;
  if (K > cap_K || M > cap_M) return -2;
  int64_t at = 0;
  c_indptr[0] = 0;
  for (int64_t s = 0; s < K; ++s) {
    const int64_t v = order[(size_t)s];
    for (int64_t e = indptr[v]; e < indptr[v + 1]; ++e) c_indices[at++] = indices[e];
    c_indptr[s + 1] = at;
  }
  return 0;
}

// Adjacency-cache fill, element-granular (Algorithm 1 and Fig. 6 as printed).  Inputs as above plus
// the per-element access counts edge_count[E]; `indices` is rewritten in place.
//   * volume <= C_adj: everything is cached verbatim and nothing is reordered (the algorithm's first branch);
//   * otherwise node totals are the sums of the element counts; nodes are ordered by total descending
//     (ties: ascending id); inside EVERY node the elements are reordered by their own count descending
//     (ties: original order) - the listing's second loop, whose printed statement repeats the node sort, is
//     read as this per-node sort (Fig. 6: node 0's elements 4, 6, 7 become 7, 6, 4);
//   * the cache takes the longest prefix of the reorganised element stream that fits: whole nodes cost
//     8*deg + 8 bytes each (plus 8 for the leading pointer entry), and the first node that does not fit
//     contributes as many leading elements as the rest of the budget pays for (8 + 8*len, len >= 1).
// The reordering is applied to the host structure too (indices, in place), so that position p of a node
// means the same neighbour whether it is read from the cache or from the host.
// partial_node / partial_deg: the node cached in part and its full length, or -1 / 0.
// *K_out counts the cached slots including the partial one; c_indptr has *K_out + 1 entries.
int32_t oracle_fill_adj_element(int64_t N, const int64_t* indptr, int64_t* indices, const uint32_t* edge_count,
                                uint64_t C_adj, int32_t* adj_remap, int64_t* c_indptr, int64_t cap_K,
                                int64_t* c_indices, int64_t cap_M, int64_t* K_out, int64_t* M_out,
                                int64_t* partial_node, int64_t* partial_deg) {
  const int64_t E = indptr[N];
  const uint64_t volume = (uint64_t)(N + 1 + E) * 8ull;
  std::vector<int64_t> order((size_t)N);
  std::iota(order.begin(), order.end(), (int64_t)0);
  int64_t K = 0, M = 0, p_node = -1, p_deg = 0, p_len = 0;
  if (volume <= C_adj) {
    K = N;
    M = E;
  } else {
    std::vector<uint64_t> totals((size_t)N, 0);
    for (int64_t v = 0; v < N; ++v)
      for (int64_t e = indptr[v]; e < indptr[v + 1]; ++e) totals[(size_t)v] += edge_count[e];
    std::stable_sort(order.begin(), order.end(),
                     [&](int64_t x, int64_t y) { return totals[(size_t)x] > totals[(size_t)y]; });
    std::vector<int64_t> perm, tmp;
    for (int64_t v = 0; v < N; ++v) {
      const int64_t s0 = indptr[v], deg = indptr[v + 1] - s0;
      perm.resize((size_t)deg);
      std::iota(perm.begin(), perm.end(), (int64_t)0);
      std::stable_sort(perm.begin(), perm.end(),
                       [&](int64_t x, int64_t y) { return edge_count[s0 + x] > edge_count[s0 + y]; });
      tmp.assign(indices + s0, indices + s0 + deg);
      for (int64_t t = 0; t < deg; ++t) indices[s0 + t] = tmp[(size_t)perm[(size_t)t]];
    }
    uint64_t used = 8;
    while (K < N) {
      const int64_t v = order[(size_t)K];
      const uint64_t cost = 8ull * (uint64_t)(indptr[v + 1] - indptr[v]) + 8ull;
      if (used + cost > C_adj) break;
      used += cost;
      M += indptr[v + 1] - indptr[v];
      ++K;
    }
    if (C_adj < 8) K = 0;
    if (K < N && C_adj >= 8 && C_adj - used >= 16) {
      p_node = order[(size_t)K];
      p_deg = indptr[p_node + 1] - indptr[p_node];
      p_len = (int64_t)((C_adj - used - 8) / 8);  // < p_deg, because the whole node did not fit
      M += p_len;
      ++K;
    }
  }
  *K_out = K;
  *M_out = M;
  *partial_node = p_node;
  *partial_deg = p_deg;
  for (int64_t v = 0; v < N; ++v) adj_remap[v] = -1;
  for (int64_t s = 0; s < K; ++s) adj_remap[order[(size_t)s]] = (int32_t)s;
  if (!c_indptr || !c_indices) return 0;
  if (K > cap_K || M > cap_M) return -2;
  int64_t at = 0;
  c_indptr[0] = 0;
  for (int64_t s = 0; s < K; ++s) {
    const int64_t v = order[(size_t)s];
    const int64_t len = v == p_node ? p_len : indptr[v + 1] - indptr[v];
    for (int64_t e = indptr[v]; e < indptr[v] + len; ++e) c_indices[at++] = indices[e];
    c_indptr[s + 1] = at;
  }
  return 0;
}

// out[i,:] = feat[ids[i],:]
void oracle_gather(const float* feat, int32_t F, const int64_t* ids, int64_t n, float* out) {
  for (int64_t i = 0; i < n; ++i)
    for (int32_t j = 0; j < F; ++j) out[i * F + j] = feat[ids[i] * F + j];
}

// The same gather routed through a feature cache: cached rows come from feat_cache, the
// others from the host matrix.  Exists so that tests can show the two routes agree.
// counts (nullable): [0] += hits, [1] += misses.
void oracle_gather_cached(const float* feat, int32_t F, const int32_t* feat_remap, const float* feat_cache,
                          const int64_t* ids, int64_t n, float* out, int64_t* counts) {
  for (int64_t i = 0; i < n; ++i) {
    const int32_t r = feat_remap[ids[i]];
    const float* row = r >= 0 ? feat_cache + (int64_t)r * F : feat + ids[i] * F;
    for (int32_t j = 0; j < F; ++j) out[i * F + j] = row[j];
    if (counts) counts[r >= 0 ? 0 : 1] += 1;
  }
}

// The same sampler routed through an adjacency cache.  A node with a slot has cached_len =
// c_indptr[slot+1] - c_indptr[slot] leading elements of its list in the cache; its full length is
// cached_len, except for the one node that may be cached in part (partial_node, full length
// partial_deg; pass -1 / 0 when there is none).  Position p is a hit iff p < cached_len (Section IV-B,
// third paragraph, 0-based) and is then read from the cache, otherwise from the host CSR.  Only the
// frontier list and the global neighbour ids are produced; tests compare them with
// oracle_sample_khop.  counts (nullable): [0] += nodes with a slot, [1] += nodes without,
// [2] += positions read from the cache, [3] += positions read from the host.
int32_t oracle_sample_hop_cached(const int64_t* indptr, const int64_t* indices, const int32_t* adj_remap,
                                 const int64_t* c_indptr, const int64_t* c_indices, int64_t partial_node,
                                 int64_t partial_deg, const int64_t* frontier, int64_t n_frontier,
                                 uint64_t batch_index, int32_t hop, int32_t fanout, uint64_t rng_seed,
                                 int64_t* row_count, int64_t* src_global, int64_t* counts) {
  std::vector<int64_t> pos((size_t)std::max(fanout, 1));
  int64_t at = 0;
  for (int64_t i = 0; i < n_frontier; ++i) {
    const int64_t v = frontier[i];
    const int32_t r = adj_remap[v];
    const int64_t cached_len = r >= 0 ? c_indptr[r + 1] - c_indptr[r] : 0;
    const int64_t deg = r < 0 ? indptr[v + 1] - indptr[v] : v == partial_node ? partial_deg : cached_len;
    const int32_t c = sample_positions(rng_seed, batch_index, hop, v, deg, fanout, pos.data());
    for (int32_t s = 0; s < c; ++s) {
      const bool hit = pos[s] < cached_len;
      src_global[at++] = hit ? c_indices[c_indptr[r] + pos[s]] : indices[indptr[v] + pos[s]];
      if (counts) counts[hit ? 2 : 3] += 1;
    }
    row_count[i] = c;
    if (counts) counts[r >= 0 ? 0 : 1] += 1;
  }
  return 0;
}

// Forward pass over the blocks of one mini-batch, all arithmetic in fp64.
// Layer l (0-based) uses block h = L-1-l; for each of the n_nodes[h] destination rows i:
//   model 0, GraphSAGE-mean: m_i = mean of x[src] over the row's sampled edges (zero vector for an
//            empty row); y_i = x_i W_self + m_i W_neigh + b;
//   model 1, GraphSAGE-sum (the aggregator Table III prints for GraphSAGE): m_i = sum instead;
//   model 2, GCN-avg (Table III): a_i = mean over node i itself and its sampled neighbours;
//            y_i = a_i W_neigh + b (one weight matrix per layer, w_self unused);
// followed by ReLU on every layer but the last.
// x_in is [n_nodes[L], dims[0]] fp32; weights are [dims[l], dims[l+1]] row-major fp32;
// logits is [n_nodes[0], dims[L]] fp64.
void oracle_gnn_forward(int32_t model, int32_t n_layers, const int64_t* n_nodes, const int64_t* const* blk_indptr,
                        const int32_t* const* blk_src, const float* x_in, const int32_t* dims,
                        const float* const* w_self, const float* const* w_neigh, const float* const* bias,
                        double* logits) {
  const int32_t L = n_layers;
  std::vector<double> x((size_t)(n_nodes[L] * dims[0]));
  for (size_t i = 0; i < x.size(); ++i) x[i] = (double)x_in[i];
  for (int32_t l = 0; l < L; ++l) {
    const int32_t h = L - 1 - l;
    const int64_t n_dst = n_nodes[h];
    const int32_t D = dims[l], Do = dims[l + 1];
    std::vector<double> y((size_t)(n_dst * Do));
    std::vector<double> m((size_t)D);
    for (int64_t i = 0; i < n_dst; ++i) {
      const double* xi = &x[(size_t)i * D];
      const int64_t e0 = blk_indptr[h][i], e1 = blk_indptr[h][i + 1];
      for (int32_t j = 0; j < D; ++j) m[j] = model == 2 ? xi[j] : 0.0;
      for (int64_t e = e0; e < e1; ++e) {
        const double* xs = &x[(size_t)blk_src[h][e] * D];
        for (int32_t j = 0; j < D; ++j) m[j] += xs[j];
      }
      const double denom = model == 0 ? (double)(e1 - e0) : model == 2 ? (double)(e1 - e0 + 1) : 1.0;
      if (denom > 0.0)
        for (int32_t j = 0; j < D; ++j) m[j] /= denom;
      double* yi = &y[(size_t)i * Do];
      for (int32_t o = 0; o < Do; ++o) yi[o] = (double)bias[l][o];
      for (int32_t j = 0; j < D; ++j)
        for (int32_t o = 0; o < Do; ++o) {
          if (model != 2) yi[o] += xi[j] * (double)w_self[l][(size_t)j * Do + o];
          yi[o] += m[j] * (double)w_neigh[l][(size_t)j * Do + o];
        }
      if (l != L - 1)
        for (int32_t o = 0; o < Do; ++o)
          if (yi[o] < 0.0) yi[o] = 0.0;
    }
    x.swap(y);
  }
  std::copy(x.begin(), x.begin() + (size_t)(n_nodes[0] * dims[L]), logits);
}

void oracle_sage_forward(int32_t n_layers, const int64_t* n_nodes, const int64_t* const* blk_indptr,
                         const int32_t* const* blk_src, const float* x_in, const int32_t* dims,
                         const float* const* w_self, const float* const* w_neigh, const float* const* bias,
                         double* logits) {
  oracle_gnn_forward(0, n_layers, n_nodes, blk_indptr, blk_src, x_in, dims, w_self, w_neigh, bias, logits);
}

// Whole batches on several host threads, for the benchmark's "oracle on all host cores" figure.
// Batch k of the range [first_batch, first_batch + n_batches) is run - sample, gather, forward, with
// exactly the functions above - by thread k mod n_threads.  Batches are independent units (Section V-B
// sums the three stages over the test batches) and the sampler's random numbers are a pure function of
// (seed, batch, hop, node, slot), so the order and the number of threads change nothing in any result.
// out[0] wall seconds, out[1..3] seconds spent sampling / gathering / in the forward pass summed over
// the threads, out[4] sampled edges, out[5] input rows, out[6] batches run, out[7] sum of all logits (so
// that no stage can be optimised away; also a cheap cross-check between thread counts).
int32_t oracle_run_batches(const int64_t* indptr, const int64_t* indices, const float* feat, int32_t F,
                           const int64_t* seeds, int64_t n_seeds, int32_t batch_size, int64_t first_batch,
                           int64_t n_batches, const int32_t* fanouts, int32_t n_hops, uint64_t rng_seed,
                           int32_t model, const int32_t* dims, const float* const* w_self,
                           const float* const* w_neigh, const float* const* bias, int32_t n_threads,
                           double* out) {
  if (n_threads < 1 || batch_size < 1 || n_batches < 0 || first_batch < 0 || n_hops < 1) return -1;
  typedef std::chrono::steady_clock clock;
  auto seconds = [](clock::time_point a, clock::time_point b) { return std::chrono::duration<double>(b - a).count(); };
  std::vector<std::vector<double>> acc((size_t)n_threads, std::vector<double>(8, 0.0));
  auto worker = [&](int32_t t) {
    std::vector<double>& a = acc[(size_t)t];
    for (int64_t k = t; k < n_batches; k += n_threads) {
      const int64_t b = first_batch + k;
      const int64_t lo = b * batch_size;
      if (lo >= n_seeds) break;
      const int64_t n = std::min<int64_t>(batch_size, n_seeds - lo);
      const auto t0 = clock::now();
      Batch blk;
      sample_batch(indptr, indices, seeds + lo, n, (uint64_t)b, fanouts, n_hops, rng_seed, &blk);
      const auto t1 = clock::now();
      std::vector<float> x(blk.nodes.size() * (size_t)F);
      oracle_gather(feat, F, blk.nodes.data(), (int64_t)blk.nodes.size(), x.data());
      const auto t2 = clock::now();
      std::vector<const int64_t*> bi((size_t)n_hops);
      std::vector<const int32_t*> bs((size_t)n_hops);
      for (int32_t h = 0; h < n_hops; ++h) {
        bi[(size_t)h] = blk.blk_indptr[(size_t)h].data();
        bs[(size_t)h] = blk.blk_src[(size_t)h].data();
        a[4] += (double)blk.blk_src[(size_t)h].size();
      }
      std::vector<double> logits((size_t)(n * dims[n_hops]));
      oracle_gnn_forward(model, n_hops, blk.n_nodes.data(), bi.data(), bs.data(), x.data(), dims, w_self, w_neigh, bias,
                         logits.data());
      const auto t3 = clock::now();
      a[1] += seconds(t0, t1);
      a[2] += seconds(t1, t2);
      a[3] += seconds(t2, t3);
      a[5] += (double)blk.nodes.size();
      a[6] += 1.0;
      for (double v : logits) a[7] += v;
    }
  };
  const auto w0 = clock::now();
  std::vector<std::thread> pool;
  for (int32_t t = 1; t < n_threads; ++t) pool.emplace_back(worker, t);
  worker(0);
  for (auto& th : pool) th.join();
  for (int i = 0; i < 8; ++i) out[i] = 0.0;
  out[0] = seconds(w0, clock::now());
  for (int32_t t = 0; t < n_threads; ++t)
    for (int i = 1; i < 8; ++i) out[i] += acc[(size_t)t][(size_t)i];
  return 0;
}

}  // extern "C"
