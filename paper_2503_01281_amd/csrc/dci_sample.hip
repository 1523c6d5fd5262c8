// Cache-aware multi-hop neighbour sampling, mini-batch block construction and pre-sampling
// access counting (Section II-C; Section IV; Section IV-B, first and third paragraphs).
//
// One batch is one clear of the batch's hash table, two kernels per hop and one closing kernel:
//   k_sample_hop  - one lane group per frontier node (a whole wavefront for fan-outs above 32, a
//                   half / quarter / eighth for smaller ones): read the node's list bounds from the
//                   adjacency cache or the host CSR (a position is served by the cache iff it lies
//                   below the node's cached length, which is the whole list for every node but the
//                   one an element-granular fill may have cached in part), draw the positions (Floyd's subset algorithm
//                   on Philox4x32-10, one lane per slot), read the neighbour ids, store them at the
//                   padded position row*fanout + slot and register every id in the hash table with
//                   an atomic minimum over that padded position.  A row's list bounds are noted for the
//                   batch's later hops, which sample the same row again and then need neither the slot
//                   look-up nor - for a miss - a second trip over the host link.  At hop 0 the same kernel turns
//                   the seeds into F_0; at later hops its first workgroups write the previous
//                   hop's edge ids, whose inputs are final by then.
//   k_relabel_hop - a lane is the "first appearance" of its node iff the table still holds its own
//                   padded position.  Counts them per row, prefix-sums edge counts and first
//                   appearances over all rows (chained scan with decoupled look-back), appends the
//                   first appearances to the frontier in (row, slot) order, publishes their
//                   local ids in the table and writes them as those edges' ids.
//   k_write_src   - the last hop's remaining edge ids, the batch sizes for the host, and the totals of
//                   the batch's statistics.
// Should a tile of the scan ever give up waiting for its predecessors, the batch is voided: a status
// word makes the batch's remaining kernels return at once, k_write_src zeroes the batch's sizes and
// raises the context's host flag, and the next dci_sync reports it.
// A table word holds the node id in its high half and, in its low half, either a final local id
// (below 2^31) or 2^31 + the smallest padded position seen so far, so one atomic minimum serves
// both "already in the frontier" and "who came first".
#include "dci_internal.h"

namespace dci {

// One 64-bit word per table entry: node id in the high half, value in the low half, all ones =
// empty.  Node ids are below 2^31, so a real entry is always smaller than the empty word.
typedef unsigned long long HashEntry;

constexpr unsigned int kTentative = 0x80000000u;
constexpr HashEntry kEmptyEntry = ~0ull;
constexpr int kBlock = 256;
// row_cnt[i]: bits 0..7 sampled edges of row i; bits 8..15 how many of them were read from the host although
// the node has a cache slot (only the node cached in part has any); bits 16..22 the distinct 128-byte lines
// of graph->indices the row read, bits 23..24 those of graph->indptr (both only counted when statistics are
// on); bit 30 set if the node has a slot
constexpr int kRowHitBit = 1 << 30;
constexpr int kRowCntMask = 0xFF;
constexpr int kRowHostShift = 8;
constexpr int kRowLinesShift = 16;
constexpr int kRowLinesMask = 0x7F;
constexpr int kRowBoundLinesShift = 23;
constexpr int kRowBoundLinesMask = 0x3;
constexpr int kHostLineLog2 = 7;  // the host link moves 128-byte lines: smaller reads cost a whole request each
// Batch status word (in the region that the per-batch clear fills with ones): all ones = fine; anything
// else = a relabel tile gave up waiting for its predecessors, the batch's outputs are void.
constexpr unsigned kBatchOk = 0xFFFFFFFFu;

__device__ __forceinline__ unsigned entry_val(const HashEntry* table, unsigned slot) {
  return reinterpret_cast<const unsigned*>(table)[2 * (size_t)slot];  // low half (little endian)
}
__device__ __forceinline__ void entry_set_val(HashEntry* table, unsigned slot, unsigned v) {
  reinterpret_cast<unsigned*>(table)[2 * (size_t)slot] = v;
}

// ---- Philox4x32-10 (Salmon et al., SC'11), counter-based ---------------------------------
__device__ __forceinline__ unsigned long long philox_u64(unsigned c0, unsigned c1, unsigned c2, unsigned c3,
                                                         unsigned k0, unsigned k1) {
  constexpr unsigned M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const unsigned h0 = __umulhi(M0, c0), l0 = M0 * c0;
    const unsigned h1 = __umulhi(M1, c2), l1 = M1 * c2;
    c0 = h1 ^ c1 ^ k0;
    c1 = l1;
    c2 = h0 ^ c3 ^ k1;
    c3 = l0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return (unsigned long long)c0 | ((unsigned long long)c1 << 32);
}

__device__ __forceinline__ unsigned long long uniform_below(unsigned k0, unsigned k1, long long node, unsigned batch,
                                                            int hop, int slot, unsigned long long m) {
  const unsigned long long u = philox_u64((unsigned)(unsigned long long)node,
                                          (unsigned)((unsigned long long)node >> 32), batch,
                                          ((unsigned)hop << 24) | (unsigned)slot, k0, k1);
  return __umul64hi(u, m);
}

// ---- hash table -----------------------------------------------------------------------------
// Finds or creates the entry of node u (open addressing, linear probing) and lowers its value to
// v if v is smaller; returns the slot and, in *candidate, whether v may have become the entry's
// value (the slot was empty, or held a larger value when it was looked at).  A call for which that
// is false can never be the node's first appearance; the reverse need not hold.
// For an entry that already holds u, key and value move as one word, so a single 64-bit atomic
// minimum does it; an empty slot is claimed by compare-and-swap.  Values only decrease and keys
// never change, so a stale read costs a redundant atomic at most.
__device__ __forceinline__ unsigned table_insert_min(HashEntry* table, unsigned entries, long long u,
                                                     unsigned v, bool* candidate) {
  // multiplicative hash, its high 32 bits scaled to [0, entries): the table need not be a power of two
  unsigned slot = __umulhi((unsigned)(((unsigned long long)u * 0x9E3779B97F4A7C15ull) >> 32), entries);
  const HashEntry mine = ((HashEntry)u << 32) | v;
  *candidate = false;
  for (;;) {
    HashEntry w = __atomic_load_n(&table[slot], __ATOMIC_RELAXED);
    if (w == kEmptyEntry) {
      w = atomicCAS(&table[slot], kEmptyEntry, mine);
      if (w == kEmptyEntry) {
        *candidate = true;
        return slot;
      }
    }
    if ((long long)(w >> 32) == u) {
      if ((unsigned)w > v) {
        atomicMin(&table[slot], mine);
        *candidate = true;
      }
      return slot;
    }
    slot = slot + 1 == entries ? 0u : slot + 1;
  }
}

// tmp_slot encoding: s >= 0 a table slot whose value this edge may still own; -1 no edge at this
// position; kSlotDone an edge whose local id the relabel kernel has already written (it was its node's first
// appearance); any other s <= -2 the slot -2 - s of an edge that cannot be its node's first appearance.
constexpr int kSlotDone = (int)0x80000000;
__device__ __forceinline__ unsigned slot_of(int s) { return (unsigned)(s >= 0 ? s : -2 - s); }

template <int G>
__device__ __forceinline__ unsigned long long group_bits(unsigned long long ballot, int grp_in_wave) {
  if (G == 64) return ballot;
  return (ballot >> (grp_in_wave * G)) & ((1ull << (G & 63)) - 1ull);
}

// ---- kernels ----------------------------------------------------------------------------------

struct HopArgs {
  const long long* seeds;  // hop 0 only: the seeds become F_0 inside this kernel
  long long n_seeds;
  long long* nodes;
  long long* counts;
  int hop;
  int fanout;
  const long long* indptr;
  const long long* indices;
  const int* adj_remap;
  const long long* c_indptr;
  const long long* c_indices;
  long long partial_node;  // the node whose list is cached in part (-1: none) and its full length
  long long partial_deg;
  unsigned k0, k1, batch;
  long long* tmp_u;
  int* tmp_slot;
  int* row_cnt;
  HashEntry* table;
  unsigned entries;  // of the table
  unsigned* adj_count;
  unsigned* edge_count;
  // previous hop, whose edges get their local ids at the start of this kernel (hop >= 1)
  int prev_fanout;
  const int* prev_row_cnt;
  const int* prev_tmp_slot;
  const long long* prev_blk_indptr;
  int* prev_blk_src;
  int n_write_blocks;  // leading workgroups that only do the previous hop's edge ids
  const unsigned* batch_flag;  // != kBatchOk: an earlier kernel of this batch failed, do nothing
  int count_lines;             // statistics are on: count the host lines every row touches
  // List bounds of the frontier's rows, kept for the batch's later hops (F_h is a prefix of F_{h+1}, and every
  // hop samples all of its frontier): row i -> (start in the array that serves it, length | served-by-cache << 62),
  // or a negative second word for the one node cached in part, whose bounds are looked up again.
  long long* row_memo;
  int last_hop;                // no later hop will read what this one would note
};

// blk_src of a finished hop: every edge reads the (by now final) local id of its source.
// One thread per padded position row * fanout + slot.
__device__ __forceinline__ void write_block_sources(long long n_rows, int fanout, const int* __restrict__ row_cnt,
                                                    const int* __restrict__ tmp_slot,
                                                    const long long* __restrict__ blk_indptr,
                                                    const HashEntry* table, int* __restrict__ blk_src,
                                                    int block, int n_blocks) {
  const long long total = n_rows * fanout;
  for (long long q = block * (long long)blockDim.x + threadIdx.x; q < total; q += (long long)n_blocks * blockDim.x) {
    const long long i = q / fanout;
    const int s = (int)(q - i * fanout);
    if (s < (row_cnt[i] & kRowCntMask)) {
      const int ts = tmp_slot[q];
      if (ts != kSlotDone) blk_src[blk_indptr[i] + s] = (int)entry_val(table, slot_of(ts));
    }
  }
}

// Closing kernel of a batch: the last hop's edge ids, and the batch sizes for the host.
// Hit statistics of a batch: every relabel tile leaves (rows with a cache slot, edges read from the cache) in
// its hop's array of partial sums; the closing kernel adds them up and updates the caller's counters with
// one atomic each.  (Per-tile atomics on the same few words cost 12 us per batch on a 56 k-row frontier.)
constexpr int kStatPartWords = 4;  // per relabel tile: rows with a slot, edges from the cache, lines of ids, lines of bounds
struct StatFold {
  unsigned long long* stats;                    // nullptr: no statistics
  const unsigned long long* part[DCI_MAX_HOPS]; // [kStatPartWords * tiles] per hop
  int tile_rows[DCI_MAX_HOPS];
  int n_hops;
};

__global__ __launch_bounds__(kBlock) void k_write_src(const long long* counts, int hop, int fanout,
                                                      const int* row_cnt, const int* tmp_slot,
                                                      const long long* blk_indptr, const HashEntry* table,
                                                      int* blk_src, long long* counts_host, StatFold sf,
                                                      const unsigned* batch_flag, long long* counts_rw,
                                                      unsigned* host_flag) {
  if (*batch_flag != kBatchOk) {
    // A relabel tile timed out: the batch is void.  Its sizes are zeroed so that whatever consumes the
    // batch next (gather, forward) finds nothing to do, and the context's host flag is raised for dci_sync.
    if (blockIdx.x == 0 && threadIdx.x < 2 * DCI_MAX_HOPS + 1) {
      counts_rw[threadIdx.x] = 0;
      if (counts_host) counts_host[threadIdx.x] = 0;
      if (threadIdx.x == 0) *host_flag = 1u;
    }
    return;
  }
  write_block_sources(counts[hop], fanout, row_cnt, tmp_slot, blk_indptr, table, blk_src, (int)blockIdx.x,
                      (int)gridDim.x);
  if (counts_host && blockIdx.x == 0 && threadIdx.x < 2 * DCI_MAX_HOPS + 1)
    counts_host[threadIdx.x] = counts[threadIdx.x];  // pinned host memory, visible once the stream is idle
  if (sf.stats && blockIdx.x == gridDim.x - 1) {
    __shared__ unsigned long long s_r[kBlock / kWave], s_e[kBlock / kWave];
    __shared__ unsigned long long s_l[kBlock / kWave], s_b[kBlock / kWave];
    unsigned long long hr = 0, he = 0, hl = 0, hb = 0, rows = 0, edges = 0;
    for (int h = 0; h < sf.n_hops; ++h) {
      const long long n_rows = counts[h];
      const long long n_tiles = (n_rows + sf.tile_rows[h] - 1) / sf.tile_rows[h];
      for (long long t = threadIdx.x; t < n_tiles; t += kBlock) {
        hr += sf.part[h][kStatPartWords * t];
        he += sf.part[h][kStatPartWords * t + 1];
        hl += sf.part[h][kStatPartWords * t + 2];
        hb += sf.part[h][kStatPartWords * t + 3];
      }
      rows += (unsigned long long)n_rows;
      edges += (unsigned long long)counts[DCI_MAX_HOPS + 1 + h];
    }
    hr = wave_sum_u64(hr);
    he = wave_sum_u64(he);
    hl = wave_sum_u64(hl);
    hb = wave_sum_u64(hb);
    if (lane_id() == 0) {
      s_r[threadIdx.x / kWave] = hr;
      s_e[threadIdx.x / kWave] = he;
      s_l[threadIdx.x / kWave] = hl;
      s_b[threadIdx.x / kWave] = hb;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      hr = 0;
      he = 0;
      hl = 0;
      hb = 0;
      for (int w = 0; w < kBlock / kWave; ++w) {
        hr += s_r[w];
        he += s_e[w];
        hl += s_l[w];
        hb += s_b[w];
      }
      if (edges) atomicAdd(&sf.stats[DCI_STAT_EDGES_SAMPLED], edges);
      if (hr) atomicAdd(&sf.stats[DCI_STAT_ADJ_NODE_HITS], hr);
      if (rows - hr) atomicAdd(&sf.stats[DCI_STAT_ADJ_NODE_MISSES], rows - hr);
      if (he) atomicAdd(&sf.stats[DCI_STAT_ADJ_EDGE_HITS], he);
      if (edges - he) atomicAdd(&sf.stats[DCI_STAT_ADJ_EDGE_MISSES], edges - he);
      atomicAdd(&sf.stats[DCI_STAT_INPUT_NODES], (unsigned long long)counts[sf.n_hops]);
      // a frontier node costs its pair of list bounds (16 bytes), a sampled edge its neighbour id (8 bytes),
      // charged to the tier that served them
      if (hr | he) atomicAdd(&sf.stats[DCI_STAT_BYTES_HBM], 16ull * hr + 8ull * he);
      if ((rows - hr) | (edges - he)) atomicAdd(&sf.stats[DCI_STAT_BYTES_HOST], 16ull * (rows - hr) + 8ull * (edges - he));
      if (hl) atomicAdd(&sf.stats[DCI_STAT_LINES_IDS], hl);
      if (hb) atomicAdd(&sf.stats[DCI_STAT_LINES_BOUNDS], hb);
    }
  }
}

// Phase 1 of a hop.  INIT (hop 0): row i first turns seed i into frontier entry i (final local id
// i in the table; an atomic minimum, so it also wins against a neighbour lane that registered
// the same node a moment earlier).  Otherwise the kernel starts by finishing the previous hop
// (write_block_sources), which only needs values that are already final.
template <int G, bool COUNT, bool INIT>
__global__ __launch_bounds__(kBlock) void k_sample_hop(HopArgs a) {
  const long long n_rows = INIT ? a.n_seeds : a.counts[a.hop];
  const long long n_noted = INIT ? 0 : a.counts[a.hop - 1];  // rows below this were rows of the previous hop as well
  if (INIT) {
    if (blockIdx.x == 0 && threadIdx.x == 0) a.counts[0] = a.n_seeds;
  } else if (*a.batch_flag != kBatchOk) {
    return;  // an earlier relabel tile gave up: the closing kernel voids the batch
  } else if ((int)blockIdx.x < a.n_write_blocks) {
    // the first few workgroups finish the previous hop while the others sample this one
    write_block_sources(a.counts[a.hop - 1], a.prev_fanout, a.prev_row_cnt, a.prev_tmp_slot, a.prev_blk_indptr,
                        a.table, a.prev_blk_src, (int)blockIdx.x, a.n_write_blocks);
    return;
  }
  const int block = (int)blockIdx.x - (INIT ? 0 : a.n_write_blocks);
  const int n_blocks = (int)gridDim.x - (INIT ? 0 : a.n_write_blocks);
  const int lane = lane_id();
  const int gl = lane & (G - 1);
  const int grp_in_wave = lane / G;
  constexpr int kGroups = kBlock / G;
  const int grp_in_block = (int)threadIdx.x / G;
  const int f = a.fanout;

  for (long long base = (long long)block * kGroups; base < n_rows; base += (long long)n_blocks * kGroups) {
    const long long i = base + grp_in_block;
    const bool row_ok = i < n_rows;
    long long v = 0, start = 0, d = 0, cached_len = 0;
    const long long* list = a.indices;
    bool hit = false, noted = false;
    if (row_ok) {
      if (INIT) {
        v = a.seeds[i];
        if (gl == 0) {
          a.nodes[i] = v;
          bool ignored;
          (void)table_insert_min(a.table, a.entries, v, (unsigned)i, &ignored);
        }
      } else {
        v = a.nodes[i];
      }
      if (!INIT && i < n_noted) {
        const long long m = a.row_memo[2 * i + 1];
        if (m >= 0) {
          noted = true;
          start = a.row_memo[2 * i];
          hit = (m >> 62) != 0;
          d = cached_len = m & ((1ll << 62) - 1);
          if (hit) list = a.c_indices;
        }
      }
      if (!noted) {
        const int r = a.adj_remap ? a.adj_remap[v] : -1;
        hit = r >= 0;
        if (hit) {
          start = a.c_indptr[r];
          cached_len = a.c_indptr[r + 1] - start;
          d = v == a.partial_node ? a.partial_deg : cached_len;
          list = a.c_indices;
        } else {
          start = a.indptr[v];
          d = a.indptr[v + 1] - start;
        }
        if (!a.last_hop && gl == 0) {
          a.row_memo[2 * i] = start;
          a.row_memo[2 * i + 1] = v == a.partial_node ? -1ll : (d | (hit ? (1ll << 62) : 0ll));
        }
      }
    }
    const int c = d < (long long)f ? (int)d : f;
    long long pos = gl;
    const bool floyd = row_ok && d > (long long)f;
    if (__ballot(floyd) != 0ull) {
      // slot s draws t_s below j_s + 1, j_s = d - f + s; it keeps t_s unless an earlier slot
      // already holds that value, in which case it takes j_s.
      const long long j = d - f + gl;
      long long t = 0;
      if (floyd && gl < f) t = (long long)uniform_below(a.k0, a.k1, v, a.batch, a.hop, gl, (unsigned long long)(j + 1));
      long long S = t;
      for (int s = 1; s < f; ++s) {
        const long long ts = __shfl(t, s, G);
        const bool match = floyd && gl < s && S == ts;
        const bool any = group_bits<G>(__ballot(match), grp_in_wave) != 0ull;
        if (gl == s && any) S = j;
      }
      if (floyd) pos = S;
    }
    const bool active = row_ok && gl < c;
    // position p of a node with a slot is served by the cache iff p < cached length (Section IV-B, third
    // paragraph); beyond it - possible only for the one node cached in part - the host list is read
    const bool from_host = active && hit && pos >= cached_len;
    const int n_host = __popcll(group_bits<G>(__ballot(from_host), grp_in_wave));
    const long long* src = from_host ? a.indices + (a.indptr[v] + pos) : list + (start + pos);
    int n_lines = 0, n_bound_lines = 0;
    if (a.count_lines) {
      // Miss-path traffic of the row in the unit a host link moves (128-byte lines): the distinct lines of
      // the neighbour ids it reads from graph->indices, and the lines its list bounds in graph->indptr lie in.
      const bool host_read = active && (from_host || !hit);
      if (__ballot(host_read) != 0ull) {
        const unsigned long long line = (unsigned long long)reinterpret_cast<uintptr_t>(src) >> kHostLineLog2;
        bool leader = host_read;
        for (int s = 0; s + 1 < f; ++s) {
          const unsigned long long ls = __shfl(line, s, G);
          const bool hs = __shfl((int)host_read, s, G) != 0;
          if (gl > s && hs && ls == line) leader = false;
        }
        n_lines = __popcll(group_bits<G>(__ballot(leader), grp_in_wave));
      }
      if (row_ok && hit && n_host > 0) n_bound_lines = 1;  // the partly cached node: where its host list starts
      if (row_ok && !hit && !noted) {  // (a noted row's bounds came from the batch's own note in HBM)
        const uintptr_t b0 = reinterpret_cast<uintptr_t>(a.indptr + v), b1 = reinterpret_cast<uintptr_t>(a.indptr + v + 1);
        n_bound_lines = (b0 >> kHostLineLog2) == (b1 >> kHostLineLog2) ? 1 : 2;
      }
    }
    if (active) {
      const long long u = *src;
      const int p = (int)(i * f + gl);
      bool candidate;
      const unsigned slot = table_insert_min(a.table, a.entries, u, kTentative | (unsigned)p, &candidate);
      a.tmp_u[p] = u;
      a.tmp_slot[p] = candidate ? (int)slot : -2 - (int)slot;  // the relabel kernel looks at the candidates only
      if (COUNT && a.edge_count) {
        const long long host_start = hit ? a.indptr[v] : start;
        atomicAdd(&a.edge_count[host_start + pos], 1u);
      }
    } else if (row_ok && gl < f) {
      a.tmp_slot[(int)(i * f + gl)] = -1;  // no edge here: lets the relabel kernel read the slots without the row count
    }
    if (row_ok && gl == 0) {
      // the hit flag rides in bit 30 so that the relabel kernel can total the hit statistics
      a.row_cnt[i] = c | (n_host << kRowHostShift) | (n_lines << kRowLinesShift) |
                     (n_bound_lines << kRowBoundLinesShift) | (hit ? kRowHitBit : 0);
      if (COUNT && c > 0) atomicAdd(&a.adj_count[v], (unsigned)c);
    }
  }
}

// Phase 2 of a hop, one pass: count the first appearances of every row, prefix-sum edge counts and
// first-appearance counts over all rows, and give the first appearances their local ids.
// The prefix sums run as a chained scan over tiles of rows with decoupled look-back: a workgroup
// takes the next tile number from a ticket counter (so every earlier tile is already running),
// publishes its own totals, and adds up its predecessors' published values until it meets one
// that already carries an inclusive prefix.  Status word: flag (2 bits) | firsts (31) | edges (31);
// the all-ones fill pattern reads as "not yet published".  A status word carries its whole
// message, so the atomic accesses are relaxed: release / acquire at device scope would add an
// L2 write-back / invalidate to every publish and every poll.
// Rows per tile = (lane groups per workgroup) x (rows per group, kTileItersMax at most).  Many rows per
// group keep several independent loads in flight per lane; few rows per group give more tiles, i.e. more
// workgroups to hide the tile's chain of dependent phases behind.  Which wins depends on how many tiles a
// frontier makes, so the count is picked per hop from the frontier's capacity (tile_iters_for).
constexpr int kTileItersMax = 8;
constexpr unsigned long long kStInvalid = 3ull, kStAggregate = 1ull, kStInclusive = 2ull;
// The look-back polls at most dci_ctx::relabel_spin_limit times (default 2^24: far beyond any real wait, ends a wedged launch).

__device__ __forceinline__ unsigned long long st_pack(unsigned long long flag, unsigned long long firsts,
                                                      unsigned long long edges) {
  return (flag << 62) | (firsts << 31) | edges;
}

struct RelabelArgs {
  long long* counts;
  int hop;
  int fanout;
  const int* row_cnt;
  const long long* tmp_u;
  int* tmp_slot;  // read; the first appearances are marked kSlotDone
  HashEntry* table;
  long long* nodes;
  long long* blk_indptr;
  int* blk_src;   // the first appearances' local ids are written here, the other edges' by the next kernel
  unsigned long long* status;  // one word per tile, filled with ones beforehand
  unsigned* ticket;            // filled with ones beforehand: the first ticket is 0xFFFFFFFF + 1 = 0
  unsigned long long* stat_part;  // [kStatPartWords * tiles] per tile, or nullptr
  unsigned* batch_flag;   // set to 0 by a tile that gives up; != kBatchOk on entry: do nothing
  unsigned spin_limit;    // polls of the look-back before a tile gives up
  unsigned first_ticket;  // tiles are numbered from here (0 except under the failure-handling test hook)
};

template <int G, int kTileIters>
__global__ __launch_bounds__(kBlock) void k_relabel_hop(RelabelArgs a) {
  constexpr int kGroups = kBlock / G;
  constexpr int TR = kGroups * kTileIters;  // rows per tile, at most kBlock
  constexpr int kWaves = kBlock / kWave;
  static_assert(TR <= kBlock, "one thread per tile row in the block scan");
  __shared__ int s_c[TR], s_f[TR];
  __shared__ int s_wc[kWaves], s_wf[kWaves];
  __shared__ unsigned long long s_hr[kWaves], s_he[kWaves], s_hl[kWaves], s_hb[kWaves];
  __shared__ unsigned s_tile;
  __shared__ long long s_ec;
  __shared__ int s_ef;
  const int tid = (int)threadIdx.x, lane = lane_id(), wave = tid / kWave;
  const int gl = lane & (G - 1), grp_in_wave = lane / G, grp = tid / G;
  if (*a.batch_flag != kBatchOk) return;  // an earlier hop failed (uniform over the launch: set before it began)
  const long long n_rows = a.counts[a.hop];
  // The grid is sized for the frontier's bound; only as many workgroups as the frontier has tiles take a
  // ticket (the tickets are atomics on one word and serialise, about 25 ns each: left to the whole grid
  // they were most of this kernel's time).  Which workgroups those are does not matter for progress: a
  // tile waits only for smaller tickets, and those are held by workgroups that are already running.
  {
    const long long n_tiles = (n_rows + TR - 1) / TR;
    long long takers = n_tiles - (long long)a.first_ticket;
    if (takers < 1) takers = 1;  // an empty frontier (or a test hook beyond it) still needs one workgroup
    if ((long long)blockIdx.x >= takers) return;
  }
  if (tid == 0) s_tile = atomicAdd(a.ticket, 1u) + 1u + a.first_ticket;
  __syncthreads();
  const unsigned tile = s_tile;
  const long long row0 = (long long)tile * TR;
  if (row0 >= n_rows) {
    // (test hook: when even the first numbered tile lies beyond the frontier nobody would notice the
    // missing tiles, so that tile voids the batch itself)
    if (a.first_ticket != 0 && tile == a.first_ticket && tid == 0)
      __hip_atomic_store(a.batch_flag, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (tile == 0 && tid == 0) {  // empty frontier: the hop adds nothing
      a.blk_indptr[0] = 0;
      a.counts[a.hop + 1] = n_rows;
      a.counts[DCI_MAX_HOPS + 1 + a.hop] = 0;
    }
    return;
  }
  const int f = a.fanout;

  // per row: sampled edges, first appearances (the table still holds the lane's own position).
  // Row counts and table slots are independent loads, the table values depend on the slots; each
  // group is issued for all of the lane's rows at once, so that the tile pays the memory latency
  // twice, not 24 times.
  int raw[kTileIters], slot[kTileIters];
  unsigned val[kTileIters];
#pragma unroll
  for (int it = 0; it < kTileIters; ++it) {
    const long long i = row0 + it * kGroups + grp;
    raw[it] = i < n_rows ? a.row_cnt[i] : 0;
  }
#pragma unroll
  for (int it = 0; it < kTileIters; ++it) {
    const long long i = row0 + it * kGroups + grp;
    slot[it] = (i < n_rows && gl < f) ? a.tmp_slot[i * f + gl] : -1;  // -1 where the row has no edge
  }
#pragma unroll
  for (int it = 0; it < kTileIters; ++it) val[it] = slot[it] >= 0 ? entry_val(a.table, (unsigned)slot[it]) : 0u;
  unsigned first_bits = 0;
  long long new_u[kTileIters];
  unsigned long long hit_rows = 0, hit_edges = 0, host_lines = 0, bound_lines = 0;
#pragma unroll
  for (int it = 0; it < kTileIters; ++it) {
    const int r = it * kGroups + grp;
    const int c = raw[it] & kRowCntMask;
    const unsigned p = (unsigned)((row0 + r) * f + gl);
    const bool first = slot[it] >= 0 && val[it] == (kTentative | p);
    const unsigned long long bits = group_bits<G>(__ballot(first), grp_in_wave);
    if (first) first_bits |= 1u << it;
    // the ids of the first appearances are only needed once the tile knows its offsets; asked for here, they
    // arrive while the tile scans and looks back
    new_u[it] = first ? a.tmp_u[(row0 + r) * f + gl] : 0;
    if (gl == 0) {
      s_c[r] = c;
      s_f[r] = __popcll(bits);
      if (raw[it] & kRowHitBit) {
        hit_rows += 1;
        hit_edges += (unsigned)(c - ((raw[it] >> kRowHostShift) & 0xFF));
      }
      host_lines += (unsigned)((raw[it] >> kRowLinesShift) & kRowLinesMask);
      bound_lines += (unsigned)((raw[it] >> kRowBoundLinesShift) & kRowBoundLinesMask);
    }
  }
  __syncthreads();

  // scan of the tile's rows, one thread per row
  const int c_t = tid < TR ? s_c[tid] : 0, f_t = tid < TR ? s_f[tid] : 0;
  const int inc_c = wave_incl_scan(c_t), inc_f = wave_incl_scan(f_t);
  if (lane == kWave - 1) {
    s_wc[wave] = inc_c;
    s_wf[wave] = inc_f;
  }
  hit_rows = wave_sum_u64(hit_rows);
  hit_edges = wave_sum_u64(hit_edges);
  host_lines = wave_sum_u64(host_lines);
  bound_lines = wave_sum_u64(bound_lines);
  if (lane == 0) {
    s_hr[wave] = hit_rows;
    s_he[wave] = hit_edges;
    s_hl[wave] = host_lines;
    s_hb[wave] = bound_lines;
  }
  __syncthreads();
  int off_c = 0, off_f = 0, tot_c = 0, tot_f = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    if (w < wave) {
      off_c += s_wc[w];
      off_f += s_wf[w];
    }
    tot_c += s_wc[w];
    tot_f += s_wf[w];
  }
  if (tid < TR) {
    s_c[tid] = off_c + inc_c;        // inclusive edge count within the tile
    s_f[tid] = off_f + inc_f - f_t;  // exclusive first-appearance count within the tile
  }

  // publish this tile, then look back over the earlier ones (first wavefront)
  if (wave == 0) {
    long long ec = 0;
    int ef = 0;
    if (tile == 0) {
      if (lane == 0)
        __hip_atomic_store(&a.status[0], st_pack(kStInclusive, (unsigned)tot_f, (unsigned)tot_c), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    } else {
      if (lane == 0)
        __hip_atomic_store(&a.status[tile], st_pack(kStAggregate, (unsigned)tot_f, (unsigned)tot_c), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
      // Look back over the earlier tiles, kLookWindows x 64 status words per round trip (lane l of window k
      // reads tile j - 64 k - l), nearest first.  A window is resolved once every word nearer than its
      // nearest inclusive one (or, if it has none, every word) is published; the sum stops at the first
      // inclusive word.
      constexpr int kLookWindows = 4;
      long long j = (long long)tile - 1;
      unsigned polls = 0;
      bool found = false, timed_out = false;
      while (!found && !timed_out) {
        unsigned long long st[kLookWindows];
#pragma unroll
        for (int k = 0; k < kLookWindows; ++k) {
          const long long idx = j - (long long)k * kWave - lane;
          st[k] = idx >= 0 ? __hip_atomic_load(&a.status[idx], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                           : st_pack(kStInclusive, 0, 0);
        }
#pragma unroll
        for (int k = 0; k < kLookWindows; ++k) {
          if (!found && !timed_out) {
            const long long idx = j - (long long)k * kWave - lane;
            int first_inc;
            for (;;) {
              const unsigned long long inv = __ballot((st[k] >> 62) == kStInvalid);
              const unsigned long long inc = __ballot((st[k] >> 62) == kStInclusive);
              first_inc = inc ? (int)__ffsll((long long)inc) - 1 : kWave;  // nearest tile with a prefix
              const unsigned long long nearer = first_inc >= kWave ? ~0ull : ((1ull << first_inc) - 1ull);
              if ((inv & nearer) == 0ull) break;
              if (polls >= a.spin_limit) {
                timed_out = true;
                break;
              }
              __builtin_amdgcn_s_sleep(1);
              ++polls;
              if ((st[k] >> 62) == kStInvalid)
                st[k] = __hip_atomic_load(&a.status[idx], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            long long pc = 0;
            int pf = 0;
            if (lane <= first_inc && (st[k] >> 62) != kStInvalid) {
              pc = (long long)(st[k] & 0x7FFFFFFFull);
              pf = (int)((st[k] >> 31) & 0x7FFFFFFFull);
            }
            ec += (long long)wave_sum_u64((unsigned long long)pc);
            ef += (int)wave_sum_u64((unsigned long long)pf);
            if (!timed_out && first_inc < kWave) found = true;
          }
        }
        j -= (long long)kLookWindows * kWave;
      }
      if (timed_out && lane == 0) {
        // Gave up: a predecessor never published.  The tile goes on with what it has - every index it
        // forms stays at or below the true one, hence inside the batch's buffers - and voids the batch,
        // so that no later kernel reads what this hop leaves behind.
        __hip_atomic_store(a.batch_flag, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      ec = __shfl(ec, 0, kWave);
      ef = __shfl(ef, 0, kWave);
      if (lane == 0)
        __hip_atomic_store(&a.status[tile], st_pack(kStInclusive, (unsigned)(ef + tot_f), (unsigned long long)(ec + tot_c)),
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (lane == 0) {
      s_ec = ec;
      s_ef = ef;
    }
  }
  __syncthreads();
  const long long ec = s_ec;
  const int ef = s_ef;
  if (tid < TR && row0 + tid < n_rows) a.blk_indptr[row0 + tid + 1] = ec + s_c[tid];

  // first appearances take the next local ids, in (row, slot) order
  long long new_id[kTileIters];
#pragma unroll
  for (int it = 0; it < kTileIters; ++it) {
    const int r = it * kGroups + grp;
    const bool first = (first_bits >> it) & 1u;
    const unsigned long long bits = group_bits<G>(__ballot(first), grp_in_wave);
    new_id[it] = first ? n_rows + ef + s_f[r] + __popcll(bits & ((1ull << gl) - 1ull)) : -1;
  }
#pragma unroll
  for (int it = 0; it < kTileIters; ++it)
    if (new_id[it] >= 0) {
      a.nodes[new_id[it]] = new_u[it];
      entry_set_val(a.table, (unsigned)slot[it], (unsigned)new_id[it]);
      // this edge's local id is known right here: write it (the row's edges sit at its sampled slots
      // 0 .. c-1, and s_c holds the row's inclusive edge count within the tile), and spare the edge-id pass
      // the table look-up
      const int r = it * kGroups + grp;
      a.blk_src[ec + s_c[r] - (raw[it] & kRowCntMask) + gl] = (int)new_id[it];
      a.tmp_slot[(row0 + r) * f + gl] = kSlotDone;
    }

  if (tid == 0) {
    if (tile == 0) a.blk_indptr[0] = 0;
    const bool last_tile = row0 + TR >= n_rows;
    if (last_tile) {
      a.counts[a.hop + 1] = n_rows + ef + tot_f;
      a.counts[DCI_MAX_HOPS + 1 + a.hop] = ec + tot_c;
    }
    if (a.stat_part) {
      unsigned long long hr = 0, he = 0, hl = 0, hb = 0;
      for (int w = 0; w < kWaves; ++w) {
        hr += s_hr[w];
        he += s_he[w];
        hl += s_hl[w];
        hb += s_hb[w];
      }
      a.stat_part[kStatPartWords * (size_t)tile] = hr;      // added up by the batch's closing kernel
      a.stat_part[kStatPartWords * (size_t)tile + 1] = he;
      a.stat_part[kStatPartWords * (size_t)tile + 2] = hl;
      a.stat_part[kStatPartWords * (size_t)tile + 3] = hb;
    }
  }
}

__global__ __launch_bounds__(kBlock) void k_count_input_nodes(const long long* __restrict__ nodes,
                                                              const long long* __restrict__ counts, int n_hops,
                                                              unsigned* __restrict__ feat_count) {
  const long long n = counts[n_hops];
  for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < n; i += (long long)gridDim.x * blockDim.x)
    atomicAdd(&feat_count[nodes[i]], 1u);
}

__global__ void k_add_u64(unsigned long long* p, unsigned long long v) { atomicAdd(p, v); }

// ---- host side ----------------------------------------------------------------------------------

struct SampleWs {
  HashEntry* table;        // the table, the tile status words and the tickets are one region,
  uint64_t table_entries;  // cleared with a single all-ones fill per batch
  unsigned long long* status[DCI_MAX_HOPS];
  unsigned* ticket;        // [DCI_MAX_HOPS]
  unsigned* batch_flag;    // one word after the tickets, also in the cleared region
  size_t clear_bytes;
  long long* tmp_u;
  int* tmp_slot[2];  // by hop parity: a hop's slots are still read while the next hop samples
  int* row_cnt[2];
  long long* row_memo;     // [2 * rows]: list bounds of the frontier's rows, noted for the batch's later hops
  unsigned long long* stat_part[DCI_MAX_HOPS];  // per hop: two words per relabel tile
};

// Twice the bound on the batch's distinct nodes (load factor at most one half), even so that the
// region is a whole number of 16-byte words for the clear.
static uint64_t table_entries_for(int64_t cap_nodes_last) {
  uint64_t want = (uint64_t)(cap_nodes_last > 0 ? cap_nodes_last : 1) * 2;
  return want < 1024 ? 1024 : want;
}

static int group_for(int fanout) { return fanout <= 8 ? 8 : fanout <= 16 ? 16 : fanout <= 32 ? 32 : 64; }

static int64_t tiles_for(int64_t rows, int fanout, int iters) {
  const int64_t tr = (int64_t)(kBlock / group_for(fanout)) * iters;
  const int64_t t = (rows + tr - 1) / tr;
  return t < 1 ? 1 : t;
}
constexpr int kTileItersMin = 2;  // the workspace is sized for the smallest tiles

// Rows per lane group of a relabel tile for a frontier of up to cap_rows rows (DCI_OPT_RELABEL_TILE_ITERS overrides).
static int tile_iters_for(const dci_ctx* ctx, int64_t cap_rows, int fanout) {
  if (ctx->relabel_tile_iters) return ctx->relabel_tile_iters;
  (void)cap_rows;
  (void)fanout;
  return kTileItersMax;
}

static void carve_sample_ws(Arena& ar, const int64_t* cap_nodes, const int64_t* cap_edges, const int32_t* fanouts,
                            int32_t n_hops, SampleWs* ws) {
  int64_t max_edges = 1, max_rows = 1;
  size_t status_words = 0;
  for (int32_t h = 0; h < n_hops; ++h) {
    if (cap_edges[h] > max_edges) max_edges = cap_edges[h];
    if (cap_nodes[h] > max_rows) max_rows = cap_nodes[h];
    status_words += (size_t)tiles_for(cap_nodes[h], fanouts[h], kTileItersMin);
  }
  ws->table_entries = table_entries_for(cap_nodes[n_hops]);
  const size_t table_bytes = ws->table_entries * sizeof(HashEntry);
  const size_t sync_bytes = align_up(status_words * 8 + (DCI_MAX_HOPS + 1) * 4, 16);
  char* region = ar.take<char>(table_bytes + sync_bytes);
  ws->table = reinterpret_cast<HashEntry*>(region);
  unsigned long long* st = reinterpret_cast<unsigned long long*>(region + table_bytes);
  for (int32_t h = 0; h < n_hops; ++h) {
    ws->status[h] = st;
    st += tiles_for(cap_nodes[h], fanouts[h], kTileItersMin);
  }
  ws->ticket = reinterpret_cast<unsigned*>(st);
  ws->batch_flag = ws->ticket + DCI_MAX_HOPS;
  ws->clear_bytes = table_bytes + sync_bytes;
  ws->tmp_u = ar.take<long long>((size_t)max_edges);
  for (int k = 0; k < 2; ++k) {
    ws->tmp_slot[k] = ar.take<int>((size_t)max_edges);
    ws->row_cnt[k] = ar.take<int>((size_t)max_rows);
  }
  ws->row_memo = ar.take<long long>(2 * (size_t)max_rows);
  for (int32_t h = 0; h < n_hops; ++h)
    ws->stat_part[h] = ar.take<unsigned long long>(kStatPartWords * (size_t)tiles_for(cap_nodes[h], fanouts[h], kTileItersMin));
}

static void carve_blocks(Arena& ar, const int64_t* cap_nodes, const int64_t* cap_edges, int32_t n_hops,
                         dci_blocks* b) {
  std::memset(b, 0, sizeof(*b));
  b->n_hops = n_hops;
  b->cap_nodes = cap_nodes[n_hops];
  b->nodes = reinterpret_cast<int64_t*>(ar.take<long long>((size_t)(cap_nodes[n_hops] > 0 ? cap_nodes[n_hops] : 1)));
  for (int32_t h = 0; h < n_hops; ++h) {
    b->cap_rows[h] = cap_nodes[h];
    b->cap_edges[h] = cap_edges[h];
    b->blk_indptr[h] = reinterpret_cast<int64_t*>(ar.take<long long>((size_t)cap_nodes[h] + 1));
    b->blk_src[h] = ar.take<int>((size_t)(cap_edges[h] > 0 ? cap_edges[h] : 1));
  }
  b->counts = reinterpret_cast<int64_t*>(ar.take<long long>(2 * DCI_MAX_HOPS + 1));
}

static int grid_for_rows(const dci_ctx* ctx, int64_t rows, int groups_per_block) {
  int64_t blocks = (rows + groups_per_block - 1) / groups_per_block;
  int64_t cap = (int64_t)ctx->num_cus * 8;
  if (blocks > cap) blocks = cap;
  if (blocks < 1) blocks = 1;
  return (int)blocks;
}

template <int G>
static int32_t launch_hop(dci_ctx* ctx, const HopArgs& ha, const RelabelArgs& ra, bool count, int64_t cap_rows) {
  const int grid = grid_for_rows(ctx, cap_rows, kBlock / G) + (ha.hop > 0 ? ha.n_write_blocks : 0);
  {
    Timed t(ctx, DCI_K_SAMPLE);
    if (ha.hop == 0) {
      if (count)
        hipLaunchKernelGGL((k_sample_hop<G, true, true>), dim3(grid), dim3(kBlock), 0, ctx->stream, ha);
      else
        hipLaunchKernelGGL((k_sample_hop<G, false, true>), dim3(grid), dim3(kBlock), 0, ctx->stream, ha);
    } else {
      if (count)
        hipLaunchKernelGGL((k_sample_hop<G, true, false>), dim3(grid), dim3(kBlock), 0, ctx->stream, ha);
      else
        hipLaunchKernelGGL((k_sample_hop<G, false, false>), dim3(grid), dim3(kBlock), 0, ctx->stream, ha);
    }
  }
  DCI_LAUNCH_CHECK(ctx);
  {
    Timed t(ctx, DCI_K_RELABEL);
    const int iters = tile_iters_for(ctx, cap_rows, ha.fanout);
    const dim3 grid_r((unsigned)tiles_for(cap_rows, ha.fanout, iters));
    if (iters == 2)
      hipLaunchKernelGGL((k_relabel_hop<G, 2>), grid_r, dim3(kBlock), 0, ctx->stream, ra);
    else if (iters == 4)
      hipLaunchKernelGGL((k_relabel_hop<G, 4>), grid_r, dim3(kBlock), 0, ctx->stream, ra);
    else
      hipLaunchKernelGGL((k_relabel_hop<G, 8>), grid_r, dim3(kBlock), 0, ctx->stream, ra);
  }
  DCI_LAUNCH_CHECK(ctx);
  return DCI_OK;
}

// Enqueues the sampling of one batch: one clear, two kernels per hop, one closing kernel.
// `adj_count` non-null turns on the pre-sampling counters.
static int32_t sample_batch(dci_ctx* ctx, const dci_graph* g, const dci_cache* cache, const int64_t* seeds,
                            int64_t n_seeds, uint64_t batch_index, const int32_t* fanouts, int32_t n_hops,
                            uint64_t rng_seed, const dci_blocks* out, const SampleWs& ws, uint64_t* stats,
                            uint32_t* feat_count, uint32_t* adj_count, uint32_t* edge_count) {
  int rc;
  {
    Timed t(ctx, DCI_K_TABLE_CLEAR);
    rc = fill_bytes(ctx, ws.table, ws.clear_bytes, 0xFFFFFFFFu);
  }
  if (rc != DCI_OK) return rc;
  long long* counts = reinterpret_cast<long long*>(out->counts);
  long long* nodes = reinterpret_cast<long long*>(out->nodes);
  const bool count = adj_count != nullptr;
  for (int32_t h = 0; h < n_hops; ++h) {
    HopArgs ha;
    ha.seeds = reinterpret_cast<const long long*>(seeds);
    ha.n_seeds = n_seeds;
    ha.nodes = nodes;
    ha.counts = counts;
    ha.hop = h;
    ha.fanout = fanouts[h];
    ha.indptr = reinterpret_cast<const long long*>(g->indptr);
    ha.indices = reinterpret_cast<const long long*>(g->indices);
    ha.adj_remap = cache ? cache->adj_remap : nullptr;
    ha.c_indptr = cache ? reinterpret_cast<const long long*>(cache->c_indptr) : nullptr;
    ha.c_indices = cache ? reinterpret_cast<const long long*>(cache->c_indices) : nullptr;
    ha.partial_node = cache ? cache->adj_partial_node : -1;
    ha.partial_deg = cache ? cache->adj_partial_deg : 0;
    ha.k0 = (unsigned)rng_seed;
    ha.k1 = (unsigned)(rng_seed >> 32);
    ha.batch = (unsigned)batch_index;
    ha.tmp_u = ws.tmp_u;
    ha.tmp_slot = ws.tmp_slot[h & 1];
    ha.row_cnt = ws.row_cnt[h & 1];
    ha.table = ws.table;
    ha.entries = (unsigned)ws.table_entries;
    ha.adj_count = adj_count;
    ha.edge_count = edge_count;
    ha.prev_fanout = h > 0 ? fanouts[h - 1] : 1;
    ha.prev_row_cnt = ws.row_cnt[(h + 1) & 1];
    ha.prev_tmp_slot = ws.tmp_slot[(h + 1) & 1];
    ha.prev_blk_indptr = h > 0 ? reinterpret_cast<const long long*>(out->blk_indptr[h - 1]) : nullptr;
    ha.prev_blk_src = h > 0 ? out->blk_src[h - 1] : nullptr;
    ha.n_write_blocks = h > 0 ? grid_for_rows(ctx, out->cap_rows[h - 1] * fanouts[h - 1], kBlock * 4) : 0;
    ha.batch_flag = ws.batch_flag;
    ha.count_lines = stats ? 1 : 0;
    ha.row_memo = ws.row_memo;
    ha.last_hop = h == n_hops - 1 ? 1 : 0;
    RelabelArgs ra;
    ra.counts = counts;
    ra.hop = h;
    ra.fanout = fanouts[h];
    ra.row_cnt = ws.row_cnt[h & 1];
    ra.tmp_u = ws.tmp_u;
    ra.tmp_slot = ws.tmp_slot[h & 1];
    ra.table = ws.table;
    ra.nodes = nodes;
    ra.blk_indptr = reinterpret_cast<long long*>(out->blk_indptr[h]);
    ra.blk_src = out->blk_src[h];
    ra.status = ws.status[h];
    ra.ticket = ws.ticket + h;
    ra.stat_part = stats ? ws.stat_part[h] : nullptr;
    ra.batch_flag = ws.batch_flag;
    ra.spin_limit = ctx->relabel_spin_limit;
    ra.first_ticket = ctx->test_first_ticket;
    // launch shapes follow the frontier bound of this call; with zero seeds one workgroup still
    // runs so that the (empty) sizes get written
    const int64_t rows = out->cap_rows[h];
    switch (group_for(fanouts[h])) {
      case 8: rc = launch_hop<8>(ctx, ha, ra, count, rows); break;
      case 16: rc = launch_hop<16>(ctx, ha, ra, count, rows); break;
      case 32: rc = launch_hop<32>(ctx, ha, ra, count, rows); break;
      default: rc = launch_hop<64>(ctx, ha, ra, count, rows); break;
    }
    if (rc != DCI_OK) return rc;
  }
  {
    const int32_t h = n_hops - 1;
    const int64_t positions = out->cap_rows[h] * fanouts[h];
    StatFold sf;
    sf.stats = reinterpret_cast<unsigned long long*>(stats);
    sf.n_hops = n_hops;
    for (int32_t k = 0; k < DCI_MAX_HOPS; ++k) {
      sf.part[k] = k < n_hops ? ws.stat_part[k] : nullptr;
      sf.tile_rows[k] = k < n_hops ? (kBlock / group_for(fanouts[k])) * tile_iters_for(ctx, out->cap_rows[k], fanouts[k]) : 1;
    }
    Timed t(ctx, DCI_K_WRITE_SRC);
    hipLaunchKernelGGL(k_write_src, dim3(grid_for_rows(ctx, positions, kBlock)), dim3(kBlock), 0, ctx->stream,
                       (const long long*)counts, h, fanouts[h], (const int*)ws.row_cnt[h & 1],
                       (const int*)ws.tmp_slot[h & 1], reinterpret_cast<const long long*>(out->blk_indptr[h]),
                       (const HashEntry*)ws.table, out->blk_src[h], reinterpret_cast<long long*>(out->counts_host), sf,
                       (const unsigned*)ws.batch_flag, counts, ctx->host_flag);
  }
  DCI_LAUNCH_CHECK(ctx);
  if (feat_count) {
    int grid = grid_for_rows(ctx, out->cap_nodes, kBlock);
    Timed t(ctx, DCI_K_COUNT_NODES);
    hipLaunchKernelGGL(k_count_input_nodes, dim3(grid), dim3(kBlock), 0, ctx->stream, (const long long*)nodes,
                       (const long long*)counts, n_hops, feat_count);
    DCI_LAUNCH_CHECK(ctx);
  }
  return DCI_OK;
}

static int32_t check_common(dci_ctx* ctx, const dci_graph* g, const int64_t* seeds, int64_t n_seeds,
                            const int32_t* fanouts, int32_t n_hops, uint64_t last_batch_index) {
  if (!g || !g->indptr || !g->indices || g->num_nodes < 1 || g->num_edges < 0)
    return fail(ctx, DCI_ERR_INVALID_ARG, "graph: null arrays or bad sizes");
  if (g->num_nodes >= ((int64_t)1 << 31)) return fail(ctx, DCI_ERR_UNSUPPORTED, "more than 2^31-1 nodes");
  if (n_seeds < 0 || (!seeds && n_seeds > 0)) return fail(ctx, DCI_ERR_INVALID_ARG, "seeds: null or negative count");
  if (!fanouts || n_hops < 1 || n_hops > DCI_MAX_HOPS)
    return fail(ctx, DCI_ERR_INVALID_ARG, "n_hops must be 1..%d", DCI_MAX_HOPS);
  for (int32_t h = 0; h < n_hops; ++h)
    if (fanouts[h] < 1 || fanouts[h] > DCI_MAX_FANOUT)
      return fail(ctx, DCI_ERR_INVALID_ARG, "fanouts[%d] = %d outside 1..%d", h, fanouts[h], DCI_MAX_FANOUT);
  if (last_batch_index >> 32) return fail(ctx, DCI_ERR_INVALID_ARG, "batch index must be below 2^32");
  return DCI_OK;
}

static int32_t check_cache(dci_ctx* ctx, const dci_cache* cache) {
  if (cache && (!cache->adj_remap || !cache->feat_remap || (cache->adj_nodes > 0 && (!cache->c_indptr || (cache->adj_edges > 0 && !cache->c_indices)))))
    return fail(ctx, DCI_ERR_INVALID_ARG, "cache: null arrays");
  return DCI_OK;
}

}  // namespace dci

using namespace dci;

extern "C" {

size_t dci_sample_workspace_bytes(int64_t num_nodes, int64_t n_seeds, const int32_t* fanouts, int32_t n_hops) {
  int64_t cap_nodes[DCI_MAX_HOPS + 1], cap_edges[DCI_MAX_HOPS];
  if (dci_blocks_bounds(num_nodes, n_seeds, fanouts, n_hops, cap_nodes, cap_edges) != DCI_OK) return 0;
  Arena ar(nullptr, 0);
  SampleWs ws;
  dci_blocks b;
  carve_sample_ws(ar, cap_nodes, cap_edges, fanouts, n_hops, &ws);
  carve_blocks(ar, cap_nodes, cap_edges, n_hops, &b);
  (void)ar.take<char>(256 * 1024);  // room for the gather statistics of the pre-sampling pass
  return ar.off;
}

// Shared body of dci_sample_khop and dci_sample_khop_static: the two differ only in where the
// temporaries live (`ws_base`, `ws_bytes`; `ws_name` names that memory in the error message).
static int32_t sample_khop_in(dci_ctx* ctx, const dci_graph* graph, const dci_cache* cache, const int64_t* seeds,
                              int64_t n_seeds, uint64_t batch_index, const int32_t* fanouts, int32_t n_hops,
                              uint64_t rng_seed, dci_blocks* out, uint64_t* stats, char* ws_base, size_t ws_bytes,
                              const char* ws_name) {
  int32_t rc = check_common(ctx, graph, seeds, n_seeds, fanouts, n_hops, batch_index);
  if (rc != DCI_OK) return rc;
  if ((rc = check_cache(ctx, cache)) != DCI_OK) return rc;
  if (!out || !out->nodes || !out->counts || out->n_hops != n_hops)
    return fail(ctx, DCI_ERR_INVALID_ARG, "blocks: null arrays or n_hops mismatch");
  int64_t cap_nodes[DCI_MAX_HOPS + 1], cap_edges[DCI_MAX_HOPS];
  rc = dci_blocks_bounds(graph->num_nodes, n_seeds, fanouts, n_hops, cap_nodes, cap_edges);
  if (rc != DCI_OK) return fail(ctx, rc, "batch bounds reach 2^31");
  {  // remembered for dci_last_required, should one of the capacity checks below fail
    Arena probe(nullptr, 0);
    SampleWs unused;
    carve_sample_ws(probe, cap_nodes, cap_edges, fanouts, n_hops, &unused);
    std::memset(ctx->req_nodes, 0, sizeof(ctx->req_nodes));
    std::memset(ctx->req_edges, 0, sizeof(ctx->req_edges));
    for (int32_t h = 0; h <= n_hops; ++h) ctx->req_nodes[h] = cap_nodes[h];
    for (int32_t h = 0; h < n_hops; ++h) ctx->req_edges[h] = cap_edges[h];
    ctx->req_workspace = probe.off;
  }
  if (out->cap_nodes < cap_nodes[n_hops])
    return fail(ctx, DCI_ERR_CAPACITY, "blocks.nodes holds %lld entries, %lld needed", (long long)out->cap_nodes,
                (long long)cap_nodes[n_hops]);
  for (int32_t h = 0; h < n_hops; ++h) {
    if (!out->blk_indptr[h] || !out->blk_src[h]) return fail(ctx, DCI_ERR_INVALID_ARG, "blocks: null array at hop %d", h);
    if (out->cap_rows[h] < cap_nodes[h] || out->cap_edges[h] < cap_edges[h])
      return fail(ctx, DCI_ERR_CAPACITY, "block %d holds %lld rows / %lld edges, %lld / %lld needed", h,
                  (long long)out->cap_rows[h], (long long)out->cap_edges[h], (long long)cap_nodes[h],
                  (long long)cap_edges[h]);
  }
  Arena ar(ws_base, ws_bytes);
  SampleWs ws;
  carve_sample_ws(ar, cap_nodes, cap_edges, fanouts, n_hops, &ws);
  if (!ar.ok())
    return fail(ctx, DCI_ERR_CAPACITY, "%s holds %zu bytes, sampling a batch of these bounds needs %zu", ws_name,
                ws_bytes, ar.off);
  // launch shapes follow the bounds of this call, not the (possibly larger) capacities
  dci_blocks view = *out;
  for (int32_t h = 0; h < n_hops; ++h) view.cap_rows[h] = cap_nodes[h];
  view.cap_nodes = cap_nodes[n_hops];
  return sample_batch(ctx, graph, cache, seeds, n_seeds, batch_index, fanouts, n_hops, rng_seed, &view, ws, stats,
                      nullptr, nullptr, nullptr);
}

int32_t dci_sample_khop(dci_ctx* ctx, const dci_graph* graph, const dci_cache* cache, const int64_t* seeds,
                        int64_t n_seeds, uint64_t batch_index, const int32_t* fanouts, int32_t n_hops,
                        uint64_t rng_seed, dci_blocks* out, uint64_t* stats) {
  if (!ctx) return DCI_ERR_INVALID_ARG;
  return sample_khop_in(ctx, graph, cache, seeds, n_seeds, batch_index, fanouts, n_hops, rng_seed, out, stats,
                        ctx->ws, ctx->ws_bytes, "workspace");
}

int32_t dci_sample_khop_static(dci_ctx* ctx, const dci_graph* graph, const dci_cache* cache, const int64_t* seeds,
                               int64_t n_seeds, uint64_t batch_index, const int32_t* fanouts, int32_t n_hops,
                               uint64_t rng_seed, dci_blocks* out, uint64_t* stats) {
  if (!ctx) return DCI_ERR_INVALID_ARG;
  if (!ctx->static_scratch) return fail(ctx, DCI_ERR_HIP, "the static scratch array has no address on this device");
  return sample_khop_in(ctx, graph, cache, seeds, n_seeds, batch_index, fanouts, n_hops, rng_seed, out, stats,
                        ctx->static_scratch, (size_t)DCI_STATIC_SCRATCH_BYTES, "the static scratch array");
}

size_t dci_sample_khop_scratch_bytes(int64_t num_nodes, int64_t n_seeds, const int32_t* fanouts, int32_t n_hops) {
  int64_t cap_nodes[DCI_MAX_HOPS + 1], cap_edges[DCI_MAX_HOPS];
  if (dci_blocks_bounds(num_nodes, n_seeds, fanouts, n_hops, cap_nodes, cap_edges) != DCI_OK) return 0;
  Arena ar(nullptr, 0);
  SampleWs ws;
  carve_sample_ws(ar, cap_nodes, cap_edges, fanouts, n_hops, &ws);
  return ar.off;
}

int32_t dci_presample_count(dci_ctx* ctx, const dci_graph* graph, const dci_cache* cache, const int64_t* seeds,
                            int64_t n_seeds, int32_t batch_size, int64_t first_batch, int64_t n_batches,
                            uint64_t rng_batch0, const int32_t* fanouts, int32_t n_hops, uint64_t rng_seed,
                            uint32_t* feat_count, uint32_t* adj_count, uint32_t* edge_count, float* feat_scratch,
                            uint64_t* stats) {
  if (!ctx) return DCI_ERR_INVALID_ARG;
  if (batch_size < 1 || first_batch < 0 || n_batches < 0)
    return fail(ctx, DCI_ERR_INVALID_ARG, "batch_size / first_batch / n_batches out of range");
  int32_t rc = check_common(ctx, graph, seeds, n_seeds, fanouts, n_hops,
                            rng_batch0 + (uint64_t)(n_batches > 0 ? n_batches - 1 : 0));
  if (rc != DCI_OK) return rc;
  if ((rc = check_cache(ctx, cache)) != DCI_OK) return rc;
  if (!feat_count || !adj_count) return fail(ctx, DCI_ERR_INVALID_ARG, "feat_count / adj_count are required");
  if (feat_scratch && !graph->feat) return fail(ctx, DCI_ERR_INVALID_ARG, "feat_scratch given but graph.feat is NULL");
  int64_t cap_nodes[DCI_MAX_HOPS + 1], cap_edges[DCI_MAX_HOPS];
  rc = dci_blocks_bounds(graph->num_nodes, batch_size, fanouts, n_hops, cap_nodes, cap_edges);
  if (rc != DCI_OK) return fail(ctx, rc, "batch bounds reach 2^31");
  Arena ar(ctx->ws, ctx->ws_bytes);
  SampleWs ws;
  dci_blocks blk;
  carve_sample_ws(ar, cap_nodes, cap_edges, fanouts, n_hops, &ws);
  carve_blocks(ar, cap_nodes, cap_edges, n_hops, &blk);
  void* gather_partials = ar.take<char>(gather_partials_bytes(ctx));
  if (!ar.ok())
    return fail(ctx, DCI_ERR_CAPACITY, "workspace holds %zu bytes, pre-sampling needs %zu", ctx->ws_bytes, ar.off);
  double ms_sample = 0.0, ms_feature = 0.0;
  for (int64_t k = 0; k < n_batches; ++k) {
    const int64_t lo = (first_batch + k) * batch_size;
    if (lo >= n_seeds) break;
    const int64_t hi = lo + batch_size < n_seeds ? lo + batch_size : n_seeds;
    if (feat_scratch) DCI_HIP(ctx, hipEventRecord(ctx->ev[0], ctx->stream));
    rc = sample_batch(ctx, graph, cache, seeds + lo, hi - lo, rng_batch0 + (uint64_t)k, fanouts, n_hops, rng_seed,
                      &blk, ws, stats, feat_count, adj_count, edge_count);
    if (rc != DCI_OK) return rc;
    if (feat_scratch) {
      DCI_HIP(ctx, hipEventRecord(ctx->ev[1], ctx->stream));
      rc = gather_launch(ctx, graph, cache, blk.nodes, cap_nodes[n_hops], blk.counts + n_hops, feat_scratch, stats,
                         gather_partials, nullptr, nullptr, 0);
      if (rc != DCI_OK) return rc;
      DCI_HIP(ctx, hipEventRecord(ctx->ev[2], ctx->stream));
      DCI_HIP(ctx, hipEventSynchronize(ctx->ev[2]));
      if ((rc = check_device_flag(ctx)) != DCI_OK) return rc;
      float a = 0.f, b = 0.f;
      DCI_HIP(ctx, hipEventElapsedTime(&a, ctx->ev[0], ctx->ev[1]));
      DCI_HIP(ctx, hipEventElapsedTime(&b, ctx->ev[1], ctx->ev[2]));
      ms_sample += a;
      ms_feature += b;
    }
  }
  if (feat_scratch && stats) {
    unsigned long long* st = reinterpret_cast<unsigned long long*>(stats);
    hipLaunchKernelGGL(k_add_u64, dim3(1), dim3(1), 0, ctx->stream, st + DCI_STAT_T_SAMPLE_NS,
                       (unsigned long long)(ms_sample * 1.0e6));
    DCI_LAUNCH_CHECK(ctx);
    hipLaunchKernelGGL(k_add_u64, dim3(1), dim3(1), 0, ctx->stream, st + DCI_STAT_T_FEATURE_NS,
                       (unsigned long long)(ms_feature * 1.0e6));
    DCI_LAUNCH_CHECK(ctx);
  }
  return DCI_OK;
}

}  // extern "C"
