// Capacity split and dual-cache fill (Eq. (1); Section IV-B; Algorithm 1: node-granular by default,
// element-granular as printed - second-level sort inside the nodes, last node cached in part - with
// DCI_FILL_ADJ_ELEMENTS).
//
// Everything that touches N-sized arrays runs on the GPU: reductions (sum / max of the
// counters), a three-kernel prefix scan, a stable LSD radix sort of (count, id) pairs for the
// orders by access count, and the bulk copies of the chosen feature rows and neighbour lists
// from (host) memory into the cache arrays.  The host only evaluates Eq. (1) and reads back a
// handful of scalars between phases, which is why dci_fill_caches waits for the GPU.
#include "dci_internal.h"

#include <type_traits>

namespace dci {

typedef unsigned long long u64;
typedef unsigned int u32;

constexpr int kFillBlock = 256;
constexpr int kScanPer = 8;
constexpr int kScanTile = kFillBlock * kScanPer;

// ---- block-wide helpers -------------------------------------------------------------------
// Exclusive prefix of `x` over the block's threads (thread order); *total = block sum.
__device__ __forceinline__ u64 block_excl_scan(u64 x, u64* smem /* blockDim/64 + 1 */, u64* total) {
  const int lane = lane_id(), wave = (int)threadIdx.x / kWave, n_waves = (int)blockDim.x / kWave;
  const u64 inc = (u64)wave_incl_scan64((long long)x);
  __syncthreads();  // smem may still be read from a previous call
  if (lane == kWave - 1) smem[wave] = inc;
  __syncthreads();
  u64 off = 0, tot = 0;
  for (int w = 0; w < n_waves; ++w) {
    const u64 s = smem[w];
    if (w < wave) off += s;
    tot += s;
  }
  *total = tot;
  return off + inc - x;
}

// ---- generic three-kernel exclusive scan over idx = 0..n-1 of in(idx) ---------------------
template <class In>
__global__ __launch_bounds__(kFillBlock) void k_tile_sums(long long n, In in, u64* __restrict__ tile_sums) {
  __shared__ u64 smem[kFillBlock / kWave + 1];
  const long long base = (long long)blockIdx.x * kScanTile + (long long)threadIdx.x * kScanPer;
  u64 s = 0;
#pragma unroll
  for (int k = 0; k < kScanPer; ++k)
    if (base + k < n) s += in(base + k);
  u64 total;
  (void)block_excl_scan(s, smem, &total);
  if (threadIdx.x == 0) tile_sums[blockIdx.x] = total;
}

// One workgroup: exclusive scan of tile_sums[0..n_tiles) in place, grand total to tile_sums[n_tiles].
__global__ __launch_bounds__(1024) void k_scan_tiles(u64* __restrict__ tile_sums, long long n_tiles) {
  __shared__ u64 smem[1024 / kWave + 1];
  u64 carry = 0;
  for (long long base = 0; base < n_tiles; base += 1024) {
    const long long idx = base + threadIdx.x;
    const u64 x = idx < n_tiles ? tile_sums[idx] : 0;
    u64 total;
    const u64 ex = block_excl_scan(x, smem, &total);
    if (idx < n_tiles) tile_sums[idx] = carry + ex;
    carry += total;
  }
  if (threadIdx.x == 0) tile_sums[n_tiles] = carry;
}

template <class In, class Out>
__global__ __launch_bounds__(kFillBlock) void k_scan_apply(long long n, In in, const u64* __restrict__ tile_sums,
                                                           Out out) {
  __shared__ u64 smem[kFillBlock / kWave + 1];
  const long long base = (long long)blockIdx.x * kScanTile + (long long)threadIdx.x * kScanPer;
  u64 v[kScanPer];
  u64 s = 0;
#pragma unroll
  for (int k = 0; k < kScanPer; ++k) {
    v[k] = base + k < n ? in(base + k) : 0;
    s += v[k];
  }
  u64 total;
  u64 run = tile_sums[blockIdx.x] + block_excl_scan(s, smem, &total);
#pragma unroll
  for (int k = 0; k < kScanPer; ++k) {
    if (base + k < n) out(base + k, run, v[k]);
    run += v[k];
  }
}

template <class In, class Out>
static int32_t device_scan(dci_ctx* ctx, long long n, In in, Out out, u64* tile_sums /* n_tiles + 1 */) {
  const long long n_tiles = (n + kScanTile - 1) / kScanTile;
  if (n_tiles > 0) {
    hipLaunchKernelGGL((k_tile_sums<In>), dim3((unsigned)n_tiles), dim3(kFillBlock), 0, ctx->stream, n, in, tile_sums);
    DCI_LAUNCH_CHECK(ctx);
  }
  hipLaunchKernelGGL(k_scan_tiles, dim3(1), dim3(1024), 0, ctx->stream, tile_sums, n_tiles);
  DCI_LAUNCH_CHECK(ctx);
  if (n_tiles > 0) {
    hipLaunchKernelGGL((k_scan_apply<In, Out>), dim3((unsigned)n_tiles), dim3(kFillBlock), 0, ctx->stream, n, in,
                       (const u64*)tile_sums, out);
    DCI_LAUNCH_CHECK(ctx);
  }
  return DCI_OK;
}

static inline long long scan_tiles_for(long long n) { return (n + kScanTile - 1) / kScanTile + 1; }

// ---- reductions -----------------------------------------------------------------------------
// scal[0] += sum(count), scal[1] = max(scal[1], max(count)), scal[3] += number of non-zero counts
__global__ __launch_bounds__(kFillBlock) void k_sum_max(const u32* __restrict__ count, long long n, u64* scal) {
  u64 s = 0, nz = 0;
  u32 m = 0;
  for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < n; i += (long long)gridDim.x * blockDim.x) {
    const u32 c = count[i];
    s += c;
    nz += c != 0;
    m = c > m ? c : m;
  }
  s = wave_sum_u64(s);
  nz = wave_sum_u64(nz);
#pragma unroll
  for (int d = kWave / 2; d >= 1; d >>= 1) {
    const u32 o = __shfl_down(m, d, kWave);
    m = o > m ? o : m;
  }
  if (lane_id() == 0) {
    if (s) atomicAdd(&scal[0], s);
    if (m) atomicMax(&scal[1], (u64)m);
    if (nz) atomicAdd(&scal[3], nz);
  }
}

// deg[v] = indptr[v+1] - indptr[v] (streaming read of the host array)
__global__ __launch_bounds__(kFillBlock) void k_degrees(const long long* __restrict__ indptr, long long n,
                                                        u32* __restrict__ deg) {
  for (long long v = blockIdx.x * (long long)blockDim.x + threadIdx.x; v < n; v += (long long)gridDim.x * blockDim.x)
    deg[v] = (u32)(indptr[v + 1] - indptr[v]);
}

// ---- stable LSD radix sort of (key, id) pairs, 8 bits per pass --------------------------------
// Keys are max_count - count, so ascending key = descending count; ids start ascending and
// the sort is stable, which gives the "ties by ascending id" rule.
constexpr int kRadixRounds = 16;
constexpr int kRadixTile = kFillBlock * kRadixRounds;

struct RadixSrc {
  const u32* keys;   // nullptr on the first pass: key = max_count - count[idx], id = idx
  const int* ids;
  const u32* count;
  u32 max_count;
  const u32* by_id;  // first pass of a re-sort of existing ids: key = by_id[ids[idx]]
  __device__ __forceinline__ void get(long long idx, u32* key, int* id) const {
    if (keys) {
      *key = keys[idx];
      *id = ids[idx];
    } else if (by_id) {
      *id = ids[idx];
      *key = by_id[*id];
    } else {
      *key = max_count - count[idx];
      *id = (int)idx;
    }
  }
};

// hist[digit * n_blocks + block] = number of keys of the block's tile with that digit
__global__ __launch_bounds__(kFillBlock) void k_radix_hist(RadixSrc src, long long n, int shift, long long n_blocks,
                                                           u32* __restrict__ hist) {
  __shared__ u32 h[256];
  h[threadIdx.x] = 0;
  __syncthreads();
  const long long base = (long long)blockIdx.x * kRadixTile;
  for (int r = 0; r < kRadixRounds; ++r) {
    const long long idx = base + r * kFillBlock + threadIdx.x;
    if (idx < n) {
      u32 key;
      int id;
      src.get(idx, &key, &id);
      atomicAdd(&h[(key >> shift) & 255u], 1u);
    }
  }
  __syncthreads();
  hist[(long long)threadIdx.x * n_blocks + blockIdx.x] = h[threadIdx.x];
}

__global__ __launch_bounds__(kFillBlock) void k_radix_scatter(RadixSrc src, long long n, int shift, long long n_blocks,
                                                              const u32* __restrict__ offsets,
                                                              u32* __restrict__ keys_out, int* __restrict__ ids_out) {
  constexpr int kWaves = kFillBlock / kWave;
  __shared__ u32 running[256];          // next free global position per digit for this tile
  __shared__ u32 wave_cnt[kWaves][256]; // per round: keys of each digit held by each wave
  const int tid = (int)threadIdx.x, lane = lane_id(), wave = tid / kWave;
  running[tid] = offsets[(long long)tid * n_blocks + blockIdx.x];
  const long long base = (long long)blockIdx.x * kRadixTile;
  for (int r = 0; r < kRadixRounds; ++r) {
#pragma unroll
    for (int w = 0; w < kWaves; ++w) wave_cnt[w][tid] = 0;
    __syncthreads();
    const long long idx = base + r * kFillBlock + tid;
    const bool ok = idx < n;
    u32 key = 0;
    int id = 0;
    if (ok) src.get(idx, &key, &id);
    const u32 digit = (key >> shift) & 255u;
    // lanes of this wave holding the same digit
    u64 peers = __ballot(ok);
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      const u64 m = __ballot((digit >> b) & 1u);
      peers &= ((digit >> b) & 1u) ? m : ~m;
    }
    const int rank = __popcll(peers & ((1ull << lane) - 1ull));
    if (ok && rank == 0) wave_cnt[wave][digit] = (u32)__popcll(peers);
    __syncthreads();
    if (ok) {
      u32 pos = running[digit] + (u32)rank;
      for (int w = 0; w < wave; ++w) pos += wave_cnt[w][digit];
      keys_out[pos] = key;
      ids_out[pos] = id;
    }
    __syncthreads();
    u32 add = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) add += wave_cnt[w][tid];
    running[tid] += add;
    __syncthreads();
  }
}

struct HistIn {
  const u32* hist;
  __device__ __forceinline__ u64 operator()(long long i) const { return hist[i]; }
};
struct HistOut {
  u32* offsets;
  __device__ __forceinline__ void operator()(long long i, u64 excl, u64) const { offsets[i] = (u32)excl; }
};

struct SortWs {
  u32* keys[2];
  int* ids[2];
  u32* hist;
  u64* tile_sums;
};

static void carve_sort_ws(Arena& ar, long long n, SortWs* ws) {
  const long long n_blocks = (n + kRadixTile - 1) / kRadixTile;
  ws->keys[0] = ar.take<u32>((size_t)n);
  ws->keys[1] = ar.take<u32>((size_t)n);
  ws->ids[0] = ar.take<int>((size_t)n);
  ws->ids[1] = ar.take<int>((size_t)n);
  ws->hist = ar.take<u32>((size_t)(256 * n_blocks));
  const long long scan_n = 256 * n_blocks > n ? 256 * n_blocks : n;
  ws->tile_sums = ar.take<u64>((size_t)scan_tiles_for(scan_n));
}

// Sorts node ids by count descending (stable).  On return *order points at the sorted ids
// (one of the workspace buffers).  max_count == 0 needs no pass: the order is the identity,
// which is materialised by one pass over digit 0 so that the caller always gets an array.
static int32_t sort_by_count_desc(dci_ctx* ctx, const u32* count, long long n, u32 max_count, const SortWs& ws,
                                  const int** order) {
  int bits = 0;
  while (bits < 32 && (max_count >> bits) != 0) ++bits;
  int passes = (bits + 7) / 8;
  if (passes < 1) passes = 1;
  const long long n_blocks = (n + kRadixTile - 1) / kRadixTile;
  RadixSrc src;
  src.keys = nullptr;
  src.ids = nullptr;
  src.count = count;
  src.max_count = max_count;
  src.by_id = nullptr;
  int cur = 0;
  for (int p = 0; p < passes; ++p) {
    const int shift = 8 * p;
    hipLaunchKernelGGL(k_radix_hist, dim3((unsigned)n_blocks), dim3(kFillBlock), 0, ctx->stream, src, n, shift,
                       n_blocks, ws.hist);
    DCI_LAUNCH_CHECK(ctx);
    HistIn in{ws.hist};
    HistOut out{ws.hist};
    int32_t rc = device_scan(ctx, 256 * n_blocks, in, out, ws.tile_sums);
    if (rc != DCI_OK) return rc;
    hipLaunchKernelGGL(k_radix_scatter, dim3((unsigned)n_blocks), dim3(kFillBlock), 0, ctx->stream, src, n, shift,
                       n_blocks, (const u32*)ws.hist, ws.keys[cur], ws.ids[cur]);
    DCI_LAUNCH_CHECK(ctx);
    src.keys = ws.keys[cur];
    src.ids = ws.ids[cur];
    cur ^= 1;
  }
  *order = src.ids;
  return DCI_OK;
}

// ---- feature cache ----------------------------------------------------------------------------
// Paper's rule: above-average nodes (count * N > total) in id order, then the others in id order.
// Stable re-sort of an id array produced by sort_by_count_desc (it lives in one of ws.ids) by
// key[id] ascending, keys below 2^key_bits.  The two stages together order ids by (key ascending,
// count descending, id ascending).
static int32_t resort_by_key(dci_ctx* ctx, const int* ids_in, const u32* key_by_id, long long n, int key_bits,
                             const SortWs& ws, const int** out) {
  const long long n_blocks = (n + kRadixTile - 1) / kRadixTile;
  const int passes = (key_bits + 7) / 8;
  RadixSrc src;
  src.keys = nullptr;
  src.ids = ids_in;
  src.count = nullptr;
  src.max_count = 0;
  src.by_id = key_by_id;
  int cur = ids_in == ws.ids[0] ? 1 : 0;  // write into the buffer the input is not in
  for (int p = 0; p < passes; ++p) {
    const int shift = 8 * p;
    hipLaunchKernelGGL(k_radix_hist, dim3((unsigned)n_blocks), dim3(kFillBlock), 0, ctx->stream, src, n, shift,
                       n_blocks, ws.hist);
    DCI_LAUNCH_CHECK(ctx);
    HistIn in{ws.hist};
    HistOut o{ws.hist};
    int32_t rc = device_scan(ctx, 256 * n_blocks, in, o, ws.tile_sums);
    if (rc != DCI_OK) return rc;
    hipLaunchKernelGGL(k_radix_scatter, dim3((unsigned)n_blocks), dim3(kFillBlock), 0, ctx->stream, src, n, shift,
                       n_blocks, (const u32*)ws.hist, ws.keys[cur], ws.ids[cur]);
    DCI_LAUNCH_CHECK(ctx);
    src.keys = ws.keys[cur];
    src.ids = ws.ids[cur];
    src.by_id = nullptr;
    cur ^= 1;
  }
  *out = src.ids;
  return DCI_OK;
}

struct AboveIn {
  const u32* count;
  const u64* scal;  // [0] = total
  u64 n;
  __device__ __forceinline__ u64 operator()(long long v) const {
    return ((u64)count[v] * n > scal[0]) ? 1u : 0u;  // count < 2^32 and n < 2^31: no overflow
  }
};
struct MeanRemapOut {
  int* remap;
  const u64* n_above;  // grand total of the scan
  long long k;
  __device__ __forceinline__ void operator()(long long v, u64 excl, u64 val) const {
    const long long pos = val ? (long long)excl : (long long)(*n_above) + (v - (long long)excl);
    remap[v] = pos < k ? (int)pos : -1;
  }
};

// remap[order[s]] = s for s < k, else -1
__global__ __launch_bounds__(kFillBlock) void k_remap_from_order(const int* __restrict__ order, long long n,
                                                                 long long k, int* __restrict__ remap) {
  for (long long s = blockIdx.x * (long long)blockDim.x + threadIdx.x; s < n; s += (long long)gridDim.x * blockDim.x)
    remap[order[s]] = s < k ? (int)s : -1;
}

// cache[remap[v], :] = feat[v, :] for every cached v; one lane group per row, source rows are
// visited in id order so that host reads stream.
template <int V>
__global__ __launch_bounds__(kFillBlock) void k_copy_rows(const int* __restrict__ remap, long long n,
                                                          const float* __restrict__ feat, int F, int lpr_log2,
                                                          float* __restrict__ cache) {
  typedef typename std::conditional<V == 4, float4, typename std::conditional<V == 2, float2, float>::type>::type vec_t;
  const int chunks = F / V;
  const int lpr = 1 << lpr_log2;
  const int rows_per_block = kFillBlock >> lpr_log2;
  const int sub = (int)threadIdx.x >> lpr_log2, cl = (int)threadIdx.x & (lpr - 1);
  for (long long base = (long long)blockIdx.x * rows_per_block; base < n; base += (long long)gridDim.x * rows_per_block) {
    const long long v = base + sub;
    if (v >= n) continue;
    const int r = remap[v];
    if (r < 0) continue;
    const vec_t* src = reinterpret_cast<const vec_t*>(feat + v * F);
    vec_t* dst = reinterpret_cast<vec_t*>(cache + (long long)r * F);
    int c = cl;
    for (; c + 3 * lpr < chunks; c += 4 * lpr) {
      const vec_t v0 = src[c], v1 = src[c + lpr], v2 = src[c + 2 * lpr], v3 = src[c + 3 * lpr];
      dst[c] = v0;
      dst[c + lpr] = v1;
      dst[c + 2 * lpr] = v2;
      dst[c + 3 * lpr] = v3;
    }
    for (; c < chunks; c += lpr) dst[c] = src[c];
  }
}

// ---- adjacency cache ----------------------------------------------------------------------------
// In sorted order s: cost = 8*deg + 8.  With P = 8 + inclusive prefix of the costs, node s is
// cached iff P <= C_adj; P is increasing, so the cached set is a prefix.
struct CostIn {
  const int* order;
  const u32* deg;
  __device__ __forceinline__ u64 operator()(long long s) const { return 8ull * deg[order[s]] + 8ull; }
};
struct AdjOut {
  const int* order;
  int* remap;
  long long* c_indptr;  // start of the region reserved for it (N+1 entries available)
  u64 c_adj;
  u64* scal;  // [2] = number of cached nodes, written by the last cached position
  const u32* deg;
  long long n;
  __device__ __forceinline__ void operator()(long long s, u64 excl, u64 cost) const {
    const u64 P = 8ull + excl + cost;
    const bool in = P <= c_adj;
    remap[order[s]] = in ? (int)s : -1;
    if (in) {
      c_indptr[s + 1] = (long long)((P - 8ull - 8ull * (u64)(s + 1)) / 8ull);
      const bool next_in = s + 1 < n && P + 8ull * deg[order[s + 1]] + 8ull <= c_adj;
      if (!next_in) scal[2] = (u64)(s + 1);
    }
  }
};

// One wavefront per cached slot s0 <= s < K copies the cached (leading) part of its node's list.
__global__ __launch_bounds__(kFillBlock) void k_copy_lists(const int* __restrict__ order, long long s0, long long K,
                                                           const long long* __restrict__ indptr,
                                                           const long long* __restrict__ indices,
                                                           const long long* __restrict__ c_indptr,
                                                           long long* __restrict__ c_indices) {
  const int lane = lane_id();
  const long long wave0 = (blockIdx.x * (long long)blockDim.x + threadIdx.x) / kWave;
  const long long n_waves = (long long)gridDim.x * blockDim.x / kWave;
  for (long long s = s0 + wave0; s < K; s += n_waves) {
    const long long v = order ? order[s] : s;
    const long long src0 = indptr[v], dst0 = c_indptr[s], len = c_indptr[s + 1] - dst0;
    long long e = lane;
    for (; e + 3 * kWave < len; e += 4 * kWave) {
      const long long a = indices[src0 + e], b = indices[src0 + e + kWave], c = indices[src0 + e + 2 * kWave],
                      d = indices[src0 + e + 3 * kWave];
      c_indices[dst0 + e] = a;
      c_indices[dst0 + e + kWave] = b;
      c_indices[dst0 + e + 2 * kWave] = c;
      c_indices[dst0 + e + 3 * kWave] = d;
    }
    for (; e < len; e += kWave) c_indices[dst0 + e] = indices[src0 + e];
  }
}

// dst[i] = src[i] (int64), streaming; used for the "whole structure fits" branch
__global__ __launch_bounds__(kFillBlock) void k_copy_i64(const long long* __restrict__ src, long long n,
                                                         long long* __restrict__ dst) {
  for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < n; i += (long long)gridDim.x * blockDim.x)
    dst[i] = src[i];
}

__global__ __launch_bounds__(kFillBlock) void k_iota_i32(int* __restrict__ p, long long n) {
  for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < n; i += (long long)gridDim.x * blockDim.x)
    p[i] = (int)i;
}

__global__ __launch_bounds__(kFillBlock) void k_fill_i32(int* __restrict__ p, long long n, int value) {
  for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < n; i += (long long)gridDim.x * blockDim.x)
    p[i] = value;
}

static int grid_1d(const dci_ctx* ctx, long long n, int per_block = kFillBlock) {
  long long b = (n + per_block - 1) / per_block;
  const long long cap = (long long)ctx->num_cus * 16;
  if (b > cap) b = cap;
  if (b < 1) b = 1;
  return (int)b;
}

// ---- element-granular mode: second-level sort inside the nodes -------------------------------
// The nodes with a non-zero total are the first n_nz of `order`; their lists, E_nz elements in all,
// are laid out one after the other (segment s at off[s]) for a stable sort by (segment, element
// count descending).  Nodes without any counted access keep their order.
struct SegLenIn {
  const int* order;
  const u32* deg;
  __device__ __forceinline__ u64 operator()(long long s) const { return deg[order[s]]; }
};
struct SegOffOut {
  long long* off;  // [n_nz + 1]
  long long n_nz;
  __device__ __forceinline__ void operator()(long long s, u64 excl, u64 len) const {
    off[s] = (long long)excl;
    if (s == n_nz - 1) off[n_nz] = (long long)(excl + len);
  }
};

// one wavefront per segment: neighbour ids (read from the host), their counts and the segment number
__global__ __launch_bounds__(kFillBlock) void k_gather_elems(const int* __restrict__ order, long long n_nz,
                                                             const long long* __restrict__ indptr,
                                                             const long long* __restrict__ indices,
                                                             const u32* __restrict__ edge_count,
                                                             const long long* __restrict__ off,
                                                             long long* __restrict__ vals, u32* __restrict__ cnt,
                                                             u32* __restrict__ seg) {
  const int lane = lane_id();
  const long long wave0 = (blockIdx.x * (long long)blockDim.x + threadIdx.x) / kWave;
  const long long n_waves = (long long)gridDim.x * blockDim.x / kWave;
  for (long long s = wave0; s < n_nz; s += n_waves) {
    const long long v = order[s];
    const long long h0 = indptr[v], o = off[s], len = off[s + 1] - o;
    for (long long t = lane; t < len; t += kWave) {
      vals[o + t] = indices[h0 + t];
      cnt[o + t] = edge_count[h0 + t];
      seg[o + t] = (u32)s;
    }
  }
}

// one wavefront per segment: the reordered list goes back to the host structure (only where it changed)
// and, for the first n_cached segments, its cached leading part into the cache
__global__ __launch_bounds__(kFillBlock) void k_scatter_elems(const int* __restrict__ order, long long n_nz,
                                                              long long n_cached,
                                                              const long long* __restrict__ indptr,
                                                              long long* __restrict__ host_indices,
                                                              const long long* __restrict__ off,
                                                              const long long* __restrict__ vals,
                                                              const int* __restrict__ sorted,
                                                              const long long* __restrict__ c_indptr,
                                                              long long* __restrict__ c_indices) {
  const int lane = lane_id();
  const long long wave0 = (blockIdx.x * (long long)blockDim.x + threadIdx.x) / kWave;
  const long long n_waves = (long long)gridDim.x * blockDim.x / kWave;
  for (long long s = wave0; s < n_nz; s += n_waves) {
    const long long v = order[s];
    const long long h0 = indptr[v], o = off[s], len = off[s + 1] - o;
    long long c0 = 0, clen = 0;
    if (s < n_cached) {
      c0 = c_indptr[s];
      clen = c_indptr[s + 1] - c0;
    }
    for (long long t = lane; t < len; t += kWave) {
      const long long j = sorted[o + t];
      const long long u = vals[j];
      if (j != o + t) host_indices[h0 + t] = u;
      if (t < clen) c_indices[c0 + t] = u;
    }
  }
}

struct ElemWs {
  long long* off;
  long long* vals;
  u32* cnt;
  u32* seg;
  SortWs sort;
};

static void carve_elem_ws(Arena& ar, long long n_nodes, long long n_elems, ElemWs* ws) {
  ws->off = ar.take<long long>((size_t)(n_nodes + 1));
  ws->vals = ar.take<long long>((size_t)n_elems);
  ws->cnt = ar.take<u32>((size_t)n_elems);
  ws->seg = ar.take<u32>((size_t)n_elems);
  carve_sort_ws(ar, n_elems > 0 ? n_elems : 1, &ws->sort);
}

struct FillWs {
  u64* scal;  // [0] sum, [1] max, [2] cached-node counter, [3] spare
  u32* deg;
  SortWs sort;
};

static void carve_fill_ws(Arena& ar, long long n, FillWs* ws) {
  ws->scal = ar.take<u64>(8);
  ws->deg = ar.take<u32>((size_t)n);
  carve_sort_ws(ar, n, &ws->sort);
}

static int32_t read_scal(dci_ctx* ctx, const u64* dev, u64* host, int n) {
  DCI_HIP(ctx, hipMemcpyAsync(host, dev, sizeof(u64) * n, hipMemcpyDeviceToHost, ctx->stream));
  DCI_HIP(ctx, hipStreamSynchronize(ctx->stream));
  return DCI_OK;
}

}  // namespace dci

using namespace dci;

extern "C" {

size_t dci_fill_workspace_bytes(int64_t num_nodes) {
  if (num_nodes < 1) return 0;
  Arena ar(nullptr, 0);
  FillWs ws;
  carve_fill_ws(ar, num_nodes, &ws);
  return ar.off;
}

size_t dci_fill_elements_workspace_bytes(int64_t num_nodes, int64_t n_elements) {
  if (num_nodes < 1 || n_elements < 0) return 0;
  Arena ar(nullptr, 0);
  FillWs ws;
  carve_fill_ws(ar, num_nodes, &ws);
  ElemWs ew;
  carve_elem_ws(ar, num_nodes, n_elements, &ew);
  return ar.off;
}

int32_t dci_fill_caches(dci_ctx* ctx, const dci_graph* g, const uint32_t* feat_count, const uint32_t* adj_count,
                        const uint32_t* edge_count, uint64_t budget_bytes, uint64_t t_sample_ns,
                        uint64_t t_feature_ns, int32_t feat_policy, void* cache_buf, int32_t* adj_remap,
                        int32_t* feat_remap, int64_t* indices_rw, dci_cache* out) {
  if (!ctx) return DCI_ERR_INVALID_ARG;
  if (!g || !g->indptr || !g->indices || !g->feat || g->num_nodes < 1 || g->num_edges < 0 || g->feat_dim < 1)
    return fail(ctx, DCI_ERR_INVALID_ARG, "graph: null arrays or bad sizes");
  if (g->num_nodes >= ((int64_t)1 << 31)) return fail(ctx, DCI_ERR_UNSUPPORTED, "more than 2^31-1 nodes");
  if (!feat_count || !adj_count || !adj_remap || !feat_remap || !out || (!cache_buf && budget_bytes > 0))
    return fail(ctx, DCI_ERR_INVALID_ARG, "fill_caches: null argument");
  const bool strict_split = (feat_policy & DCI_FILL_STRICT_SPLIT) != 0;
  const bool elements = (feat_policy & DCI_FILL_ADJ_ELEMENTS) != 0;
  feat_policy &= ~(DCI_FILL_STRICT_SPLIT | DCI_FILL_ADJ_ELEMENTS);
  if (elements && (indices_rw == nullptr || indices_rw != g->indices))
    return fail(ctx, DCI_ERR_INVALID_ARG,
                "fill_caches: the element-granular fill reorders the graph's lists in place; pass graph->indices as "
                "indices_rw to allow it");
  if (elements && !edge_count)
    return fail(ctx, DCI_ERR_INVALID_ARG, "fill_caches: DCI_FILL_ADJ_ELEMENTS needs edge_count");
  if (feat_policy != DCI_FEAT_POLICY_PAPER_MEAN && feat_policy != DCI_FEAT_POLICY_TOPK)
    return fail(ctx, DCI_ERR_INVALID_ARG, "fill_caches: unknown feature policy %d", feat_policy);
  if (reinterpret_cast<uintptr_t>(cache_buf) % kAlign)
    return fail(ctx, DCI_ERR_INVALID_ARG, "cache_buf must be %zu-byte aligned", kAlign);
  const long long N = g->num_nodes, E = g->num_edges;
  const int F = g->feat_dim;
  Arena ar(ctx->ws, ctx->ws_bytes);
  FillWs ws;
  carve_fill_ws(ar, N, &ws);
  if (!ar.ok())
    return fail(ctx, DCI_ERR_CAPACITY, "workspace holds %zu bytes, fill_caches needs %zu", ctx->ws_bytes, ar.off);

  // 1. Eq. (1) with spill-over
  const u64 C = budget_bytes;
  const u64 tsum = t_sample_ns + t_feature_ns;
  if (tsum < t_sample_ns) return fail(ctx, DCI_ERR_INVALID_ARG, "t_sample_ns + t_feature_ns overflows");
  u64 c_adj = tsum == 0 ? C / 2 : (u64)(((unsigned __int128)C * t_sample_ns) / tsum);
  u64 c_feat = C - c_adj;
  const u64 adj_total = (u64)(N + 1 + E) * 8ull, feat_total = (u64)N * (u64)F * 4ull;
  if (strict_split) {
  } else if (adj_total <= c_adj) {
    c_adj = adj_total;
    c_feat = C - adj_total;
  } else if (feat_total <= c_feat) {
    c_feat = feat_total;
    c_adj = C - feat_total;
  }
  const long long k = (long long)((c_feat / (4ull * (u64)F)) < (u64)N ? (c_feat / (4ull * (u64)F)) : (u64)N);

  char* buf = static_cast<char*>(cache_buf);
  float* feat_cache = reinterpret_cast<float*>(buf);
  const size_t adj_off = (size_t)((u64)k * (u64)F * 4ull + 7ull) / 8 * 8;
  long long* c_indptr = reinterpret_cast<long long*>(buf + adj_off);

  int32_t rc;
  auto aligned = [](const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; };

  // 2. feature cache
  if ((rc = fill_bytes(ctx, ws.scal, 64, 0u)) != DCI_OK) return rc;
  hipLaunchKernelGGL(k_sum_max, dim3(grid_1d(ctx, N)), dim3(kFillBlock), 0, ctx->stream, feat_count, N, ws.scal);
  DCI_LAUNCH_CHECK(ctx);
  if (feat_policy == DCI_FEAT_POLICY_PAPER_MEAN) {
    AboveIn in{feat_count, ws.scal, (u64)N};
    u64* tiles = ws.sort.tile_sums;
    MeanRemapOut o{feat_remap, tiles + (scan_tiles_for(N) - 1), k};
    if ((rc = device_scan(ctx, N, in, o, tiles)) != DCI_OK) return rc;
  } else {
    u64 h[2];
    if ((rc = read_scal(ctx, ws.scal, h, 2)) != DCI_OK) return rc;
    const int* order = nullptr;
    if ((rc = sort_by_count_desc(ctx, feat_count, N, (u32)h[1], ws.sort, &order)) != DCI_OK) return rc;
    hipLaunchKernelGGL(k_remap_from_order, dim3(grid_1d(ctx, N)), dim3(kFillBlock), 0, ctx->stream, order, N, k,
                       feat_remap);
    DCI_LAUNCH_CHECK(ctx);
  }
  if (k > 0) {
    int V = 1;
    if (F % 4 == 0 && aligned(g->feat, 16)) V = 4;
    else if (F % 2 == 0 && aligned(g->feat, 8)) V = 2;
    const int chunks = F / V;
    int lpr_log2 = 0;
    while ((1 << lpr_log2) < chunks && lpr_log2 < 6) ++lpr_log2;
    const int grid = grid_1d(ctx, N, kFillBlock >> lpr_log2);
    if (V == 4)
      hipLaunchKernelGGL((k_copy_rows<4>), dim3(grid), dim3(kFillBlock), 0, ctx->stream, (const int*)feat_remap, N,
                         g->feat, F, lpr_log2, feat_cache);
    else if (V == 2)
      hipLaunchKernelGGL((k_copy_rows<2>), dim3(grid), dim3(kFillBlock), 0, ctx->stream, (const int*)feat_remap, N,
                         g->feat, F, lpr_log2, feat_cache);
    else
      hipLaunchKernelGGL((k_copy_rows<1>), dim3(grid), dim3(kFillBlock), 0, ctx->stream, (const int*)feat_remap, N,
                         g->feat, F, lpr_log2, feat_cache);
    DCI_LAUNCH_CHECK(ctx);
  }

  // 3. adjacency cache
  long long K = 0, M = 0, partial_node = -1, partial_deg = 0;
  const long long* indptr = reinterpret_cast<const long long*>(g->indptr);
  const long long* indices = reinterpret_cast<const long long*>(g->indices);
  long long* c_indices = nullptr;
  if (adj_total <= c_adj) {
    K = N;
    M = E;
    c_indices = c_indptr + (K + 1);
    hipLaunchKernelGGL(k_iota_i32, dim3(grid_1d(ctx, N)), dim3(kFillBlock), 0, ctx->stream, adj_remap, N);
    DCI_LAUNCH_CHECK(ctx);
    hipLaunchKernelGGL(k_copy_i64, dim3(grid_1d(ctx, N + 1)), dim3(kFillBlock), 0, ctx->stream, indptr, N + 1, c_indptr);
    DCI_LAUNCH_CHECK(ctx);
    hipLaunchKernelGGL(k_copy_i64, dim3(grid_1d(ctx, E)), dim3(kFillBlock), 0, ctx->stream, indices, E, c_indices);
    DCI_LAUNCH_CHECK(ctx);
  } else if (c_adj < 16 && !elements) {
    // not even an empty list fits: nothing is cached
    hipLaunchKernelGGL(k_fill_i32, dim3(grid_1d(ctx, N)), dim3(kFillBlock), 0, ctx->stream, adj_remap, N, -1);
    DCI_LAUNCH_CHECK(ctx);
  } else {
    if ((rc = fill_bytes(ctx, ws.scal, 64, 0u)) != DCI_OK) return rc;
    hipLaunchKernelGGL(k_sum_max, dim3(grid_1d(ctx, N)), dim3(kFillBlock), 0, ctx->stream, adj_count, N, ws.scal);
    DCI_LAUNCH_CHECK(ctx);
    hipLaunchKernelGGL(k_degrees, dim3(grid_1d(ctx, N)), dim3(kFillBlock), 0, ctx->stream, indptr, N, ws.deg);
    DCI_LAUNCH_CHECK(ctx);
    u64 h[4];
    if ((rc = read_scal(ctx, ws.scal, h, 4)) != DCI_OK) return rc;
    const long long n_nz = (long long)h[3];  // nodes with a non-zero total: the first n_nz of the order
    const int* order = nullptr;
    if ((rc = sort_by_count_desc(ctx, adj_count, N, (u32)h[1], ws.sort, &order)) != DCI_OK) return rc;
    if (c_adj >= 16) {
      CostIn in{order, ws.deg};
      AdjOut o{order, adj_remap, c_indptr, c_adj, ws.scal, ws.deg, N};
      if ((rc = device_scan(ctx, N, in, o, ws.sort.tile_sums)) != DCI_OK) return rc;
      u64 hk[3];
      if ((rc = read_scal(ctx, ws.scal, hk, 3)) != DCI_OK) return rc;
      K = (long long)hk[2];
      // c_indptr[0] = 0, then read M = c_indptr[K]
      long long zero = 0;
      DCI_HIP(ctx, hipMemcpyAsync(c_indptr, &zero, sizeof(zero), hipMemcpyHostToDevice, ctx->stream));
      DCI_HIP(ctx, hipMemcpyAsync(&M, c_indptr + K, sizeof(M), hipMemcpyDeviceToHost, ctx->stream));
      DCI_HIP(ctx, hipStreamSynchronize(ctx->stream));
    } else {
      hipLaunchKernelGGL(k_fill_i32, dim3(grid_1d(ctx, N)), dim3(kFillBlock), 0, ctx->stream, adj_remap, N, -1);
      DCI_LAUNCH_CHECK(ctx);
    }
    if (elements && c_adj >= 16 && K < N) {
      // the first node that does not fit as a whole: its pointer entry and as many leading elements as
      // the rest of the budget pays for
      const u64 used = 8ull * (u64)(K + 1) + 8ull * (u64)M;
      if (c_adj - used >= 16) {
        int b = 0;
        u32 deg_b = 0;
        DCI_HIP(ctx, hipMemcpyAsync(&b, order + K, sizeof(b), hipMemcpyDeviceToHost, ctx->stream));
        DCI_HIP(ctx, hipStreamSynchronize(ctx->stream));
        DCI_HIP(ctx, hipMemcpyAsync(&deg_b, ws.deg + b, sizeof(deg_b), hipMemcpyDeviceToHost, ctx->stream));
        DCI_HIP(ctx, hipStreamSynchronize(ctx->stream));
        const long long len = (long long)((c_adj - used - 8ull) / 8ull);  // < deg_b: the whole node did not fit
        const int slot = (int)K;
        const long long end = M + len;
        DCI_HIP(ctx, hipMemcpyAsync(adj_remap + b, &slot, sizeof(slot), hipMemcpyHostToDevice, ctx->stream));
        DCI_HIP(ctx, hipMemcpyAsync(c_indptr + K + 1, &end, sizeof(end), hipMemcpyHostToDevice, ctx->stream));
        DCI_HIP(ctx, hipStreamSynchronize(ctx->stream));
        partial_node = b;
        partial_deg = (long long)deg_b;
        K += 1;
        M = end;
      }
    }
    c_indices = c_indptr + (K + 1);
    long long first_plain = 0;  // cached slots below this one get their lists from the element sort
    if (elements && n_nz > 0) {
      Arena ar2(ctx->ws, ctx->ws_bytes);
      FillWs ws2;
      carve_fill_ws(ar2, N, &ws2);  // same layout as ws: the element arrays follow it
      long long* off = ar2.take<long long>((size_t)(N + 1));
      if (!ar2.ok())
        return fail(ctx, DCI_ERR_CAPACITY, "workspace holds %zu bytes, the element-granular fill needs more (see dci_fill_elements_workspace_bytes)", ctx->ws_bytes);
      SegLenIn sin{order, ws.deg};
      SegOffOut sout{off, n_nz};
      // the node sort is finished with its scan scratch; `order` itself stays in use
      if ((rc = device_scan(ctx, n_nz, sin, sout, ws.sort.tile_sums)) != DCI_OK) return rc;
      long long e_nz = 0;
      DCI_HIP(ctx, hipMemcpyAsync(&e_nz, off + n_nz, sizeof(e_nz), hipMemcpyDeviceToHost, ctx->stream));
      DCI_HIP(ctx, hipStreamSynchronize(ctx->stream));
      if (e_nz >= ((long long)1 << 31))
        return fail(ctx, DCI_ERR_UNSUPPORTED, "element-granular fill: %lld list elements of counted nodes (limit 2^31-1)", e_nz);
      if (e_nz > 0) {
        Arena ar3(ctx->ws, ctx->ws_bytes);
        FillWs ws3;
        carve_fill_ws(ar3, N, &ws3);
        ElemWs ew;
        carve_elem_ws(ar3, N, e_nz, &ew);
        if (!ar3.ok())
          return fail(ctx, DCI_ERR_CAPACITY, "workspace holds %zu bytes, the element-granular fill of %lld elements needs %zu",
                      ctx->ws_bytes, e_nz, ar3.off);
        // ew.off is the array `off` carved above (same position)
        const int wpb = kFillBlock / kWave;
        hipLaunchKernelGGL(k_gather_elems, dim3(grid_1d(ctx, n_nz, wpb)), dim3(kFillBlock), 0, ctx->stream, order, n_nz,
                           indptr, indices, edge_count, (const long long*)ew.off, ew.vals, ew.cnt, ew.seg);
        DCI_LAUNCH_CHECK(ctx);
        if ((rc = fill_bytes(ctx, ws.scal, 64, 0u)) != DCI_OK) return rc;
        hipLaunchKernelGGL(k_sum_max, dim3(grid_1d(ctx, e_nz)), dim3(kFillBlock), 0, ctx->stream, (const u32*)ew.cnt, e_nz,
                           ws.scal);
        DCI_LAUNCH_CHECK(ctx);
        u64 he[2];
        if ((rc = read_scal(ctx, ws.scal, he, 2)) != DCI_OK) return rc;
        const int* by_count = nullptr;
        if ((rc = sort_by_count_desc(ctx, ew.cnt, e_nz, (u32)he[1], ew.sort, &by_count)) != DCI_OK) return rc;
        const int* sorted = by_count;
        int seg_bits = 0;
        while (seg_bits < 32 && ((u64)(n_nz - 1) >> seg_bits) != 0) ++seg_bits;
        if (seg_bits > 0 && (rc = resort_by_key(ctx, by_count, ew.seg, e_nz, seg_bits, ew.sort, &sorted)) != DCI_OK) return rc;
        const long long n_cached = n_nz < K ? n_nz : K;
        hipLaunchKernelGGL(k_scatter_elems, dim3(grid_1d(ctx, n_nz, wpb)), dim3(kFillBlock), 0, ctx->stream, order, n_nz,
                           n_cached, indptr, reinterpret_cast<long long*>(indices_rw), (const long long*)ew.off,
                           (const long long*)ew.vals, sorted, (const long long*)c_indptr, c_indices);
        DCI_LAUNCH_CHECK(ctx);
        first_plain = n_cached;
      }
    }
    if (K > first_plain) {
      // Entries of c_indptr beyond K+1 were never written; the lists start right after entry K.
      const long long waves_per_block = kFillBlock / kWave;
      hipLaunchKernelGGL(k_copy_lists, dim3(grid_1d(ctx, K - first_plain, (int)waves_per_block)), dim3(kFillBlock), 0,
                         ctx->stream, order, first_plain, K, indptr, indices, (const long long*)c_indptr, c_indices);
      DCI_LAUNCH_CHECK(ctx);
    }
  }
  DCI_HIP(ctx, hipStreamSynchronize(ctx->stream));

  std::memset(out, 0, sizeof(*out));
  out->adj_nodes = K;
  out->adj_edges = M;
  out->feat_rows = k;
  out->adj_bytes = 8ull * (u64)(K + 1) + 8ull * (u64)M;
  out->feat_bytes = 4ull * (u64)F * (u64)k;
  out->cap_adj_bytes = c_adj;
  out->cap_feat_bytes = c_feat;
  out->adj_remap = adj_remap;
  out->c_indptr = reinterpret_cast<const int64_t*>(c_indptr);
  out->c_indices = reinterpret_cast<const int64_t*>(c_indices);
  out->feat_remap = feat_remap;
  out->feat_cache = feat_cache;
  out->adj_partial_node = partial_node;
  out->adj_partial_deg = partial_deg;
  return DCI_OK;
}

}  // extern "C"
