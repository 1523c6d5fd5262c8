// Forward pass over the blocks of one mini-batch: GraphSAGE with the mean aggregator, and the two
// models of Table III (GraphSAGE with the sum aggregator, GCN with the averaging one).
//
// Per layer:
//   k_sage_mean        - m_i = mean (or sum; for GCN the mean over the row itself and its sources) of
//                        x[src] over row i of the block; bandwidth bound: one lane group per
//                        destination row, consecutive lanes on consecutive chunks of the row;
//   a dense-layer kernel - y = x W_self + m W_neigh + b (+ ReLU) (GCN: y = m W + b): one contraction
//                        over the concatenated axis on the matrix cores (v_mfma_f32_32x32x2f32, fp32 in,
//                        fp32 accumulate).  Four of them, chosen by the layer's shape (and two more,
//                        k_sage_input_res and k_sage_input_tile, that do the input layer's aggregation themselves
//                        and keep the aggregated rows out of device memory):
//       k_sage_linear_res   weights kept in registers, 32-row blocks streamed through LDS (tall layers
//                           whose whole contraction is at most 256 long, 256-column tiles);
//       k_sage_linear_wide  192x128 passes, one workgroup per compute unit, global->LDS loads
//                           (tall layers with wide inputs);
//       k_sage_linear_dma   64x64 tiles, global->LDS loads (output width a multiple of 64);
//       k_sage_linear       64x64 tiles staged through registers, any width and alignment, with the
//                           contraction split over several workgroups (+ k_split_reduce) when the
//                           layer has few tiles.
// Row counts come from the block's device-side `counts`, so no host round trip is needed; the
// grids are sized for the capacities and surplus workgroups leave at once.
#include "dci_internal.h"

#include <type_traits>

namespace dci {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kMeanBlock = 256;

template <int V>
struct VecF;
template <>
struct VecF<4> {
  typedef float4 type;
  static __device__ __forceinline__ float4 zero() { return make_float4(0.f, 0.f, 0.f, 0.f); }
  static __device__ __forceinline__ void add(float4& a, const float4& b) { a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w; }
  static __device__ __forceinline__ float4 div(const float4& a, float d) { return make_float4(a.x / d, a.y / d, a.z / d, a.w / d); }
};
template <>
struct VecF<2> {
  typedef float2 type;
  static __device__ __forceinline__ float2 zero() { return make_float2(0.f, 0.f); }
  static __device__ __forceinline__ void add(float2& a, const float2& b) { a.x += b.x; a.y += b.y; }
  static __device__ __forceinline__ float2 div(const float2& a, float d) { return make_float2(a.x / d, a.y / d); }
};
template <>
struct VecF<1> {
  typedef float type;
  static __device__ __forceinline__ float zero() { return 0.f; }
  static __device__ __forceinline__ void add(float& a, const float& b) { a += b; }
  static __device__ __forceinline__ float div(const float& a, float d) { return a / d; }
};

// REF: the input layer when cached rows are read in place - the row of source s is
// cache[rowref[s]] if rowref[s] >= 0 (its slot in the feature cache) and x[s] otherwise (a row that
// missed and was staged there); the destination's own row (GCN) is always in x.
// CPL: chunks (of V floats) per lane.  CPL >= 1: the lane keeps its CPL partial sums in registers and walks
// the row's edges once, so that an edge's source index (and cache slot) is looked up once and its row is
// read in one sweep of the lane group; CPL = 0: rows wider than 8 chunks per lane, walked chunk by chunk.
// Either way every output element adds its sources in edge order.
template <int V, bool REF, int CPL>
__global__ __launch_bounds__(kMeanBlock) void k_sage_mean(const long long* __restrict__ counts, int hop,
                                                          const long long* __restrict__ blk_indptr,
                                                          const int* __restrict__ blk_src,
                                                          const float* __restrict__ x, int D, int lpr_log2,
                                                          float* __restrict__ m, int mode,
                                                          const int* __restrict__ rowref,
                                                          const float* __restrict__ cache) {
  // mode: DCI_MODEL_SAGE_MEAN  mean of the sampled neighbours (zero vector for an empty row)
  //       DCI_MODEL_SAGE_SUM   their sum
  //       DCI_MODEL_GCN_AVG    mean over the node itself and its sampled neighbours
  typedef VecF<V> O;
  typedef typename O::type vec_t;
  const long long n_rows = counts[hop];
  const int chunks = D / V;
  const int lpr = 1 << lpr_log2;
  const int rows_per_block = kMeanBlock >> lpr_log2;
  const int sub = (int)threadIdx.x >> lpr_log2;
  const int cl = (int)threadIdx.x & (lpr - 1);
  auto row = [&](int s) -> const vec_t* {
    if (REF) {
      const int r = rowref[s];
      return reinterpret_cast<const vec_t*>(r >= 0 ? cache + (long long)r * D : x + (long long)s * D);
    }
    return reinterpret_cast<const vec_t*>(x + (long long)s * D);
  };
  for (long long base = (long long)blockIdx.x * rows_per_block; base < n_rows;
       base += (long long)gridDim.x * rows_per_block) {
    const long long i = base + sub;
    if (i >= n_rows) continue;
    const long long e0 = blk_indptr[i], e1 = blk_indptr[i + 1];
    const float cnt = (float)(e1 - e0) + (mode == DCI_MODEL_GCN_AVG ? 1.f : 0.f);
    vec_t* dst = reinterpret_cast<vec_t*>(m + i * D);
    if (CPL > 0) {
      // The launch picks CPL = ceil(chunks / lanes per row) exactly, so only a lane's last chunk can lie beyond
      // the row; such a lane reads the row's last chunk instead (in bounds, discarded), which keeps the loop
      // free of predicates.
      constexpr int N = CPL > 0 ? CPL : 1;
      constexpr int EU = N <= 2 ? 4 : 2;  // edges in flight: 8 to 16 loads per lane
      const bool last_ok = cl + (N - 1) * lpr < chunks;
      int col[N];
#pragma unroll
      for (int k = 0; k < N; ++k) col[k] = cl + k * lpr;
      if (!last_ok) col[N - 1] = chunks - 1;
      vec_t acc[N];
#pragma unroll
      for (int k = 0; k < N; ++k)
        acc[k] = mode == DCI_MODEL_GCN_AVG ? reinterpret_cast<const vec_t*>(x + i * D)[col[k]] : O::zero();
      long long e = e0;
      for (; e + EU <= e1; e += EU) {
        const vec_t* p[EU];
#pragma unroll
        for (int u = 0; u < EU; ++u) p[u] = row(blk_src[e + u]);
        vec_t v[EU][N];
#pragma unroll
        for (int u = 0; u < EU; ++u)
#pragma unroll
          for (int k = 0; k < N; ++k) v[u][k] = p[u][col[k]];
#pragma unroll
        for (int u = 0; u < EU; ++u)
#pragma unroll
          for (int k = 0; k < N; ++k) O::add(acc[k], v[u][k]);
      }
      for (; e < e1; ++e) {
        const vec_t* p = row(blk_src[e]);
#pragma unroll
        for (int k = 0; k < N; ++k) O::add(acc[k], p[col[k]]);
      }
#pragma unroll
      for (int k = 0; k < N; ++k)
        if (k < N - 1 || last_ok) dst[col[k]] = (mode == DCI_MODEL_SAGE_SUM || cnt == 0.f) ? acc[k] : O::div(acc[k], cnt);
      continue;
    }
    for (int c = cl; c < chunks; c += lpr) {
      vec_t acc = mode == DCI_MODEL_GCN_AVG ? reinterpret_cast<const vec_t*>(x + i * D)[c] : O::zero();
      long long e = e0;
      for (; e + 3 < e1; e += 4) {
        const vec_t v0 = row(blk_src[e])[c];
        const vec_t v1 = row(blk_src[e + 1])[c];
        const vec_t v2 = row(blk_src[e + 2])[c];
        const vec_t v3 = row(blk_src[e + 3])[c];
        O::add(acc, v0);
        O::add(acc, v1);
        O::add(acc, v2);
        O::add(acc, v3);
      }
      for (; e < e1; ++e) O::add(acc, row(blk_src[e])[c]);
      dst[c] = (mode == DCI_MODEL_SAGE_SUM || cnt == 0.f) ? acc : O::div(acc, cnt);
    }
  }
}

// ---- dense layer on the matrix cores ---------------------------------------------------------
// y[M, N] = a_self[M, K] w_self[K, N] + a_neigh[M, K] w_neigh[K, N] + bias, i.e. one contraction
// over the concatenated axis of length 2K.  M is read from device memory.
//
// k_sage_linear: 64x64 outputs per workgroup of four wavefronts, each wavefront one 32x32 MFMA tile
// (v_mfma_f32_32x32x2f32: lane l feeds A[l%32][l/32] and B[l/32][l%32]).  Operands go global ->
// registers -> LDS (k-major, so fragment reads hit consecutive banks) with the next k-slab in
// flight while the current one is used; every load is masked, so any width and alignment works.
// Workgroup ids are mapped so that the column tiles of one row tile run on the same XCD and
// share its L2.
constexpr int TM = 64, TN = 64, TK = 16, LDS_PAD = 4;
constexpr int kGemmThreads = 256;

struct LinearArgs {
  const long long* counts;  // M = counts[hop]
  int hop;
  const float* a_self;   // [M, K] row stride K
  const float* a_neigh;  // [M, K]
  const float* w_self;   // [K, N] row-major
  const float* w_neigh;  // [K, N]
  const float* bias;     // [N]
  float* y;              // [M, N]
  int K, N, relu;
  int n_tiles_n;
  int single;  // 1: only the (a_neigh, w_neigh) pair is used (GCN)
  // split of the contraction over several workgroups per tile (tile kernel only; 1 = no split)
  int split;            // workgroups per tile
  int n_tiles;          // tiles in the launch (= workgroups / split)
  long long part_rows;  // row capacity of one partial-sum plane
  float* part;          // [split][part_rows][N] partial sums
};

// VA: floats per global access along K for the activations (needs K % VA == 0 and aligned bases)
// VB: floats per global access along N for the weights (needs N % VB == 0)
template <int VA, int VB>
__global__ __launch_bounds__(kGemmThreads, 6) void k_sage_linear(LinearArgs a) {
  __shared__ __attribute__((aligned(16))) float As[2][TK][TM + LDS_PAD];
  __shared__ __attribute__((aligned(16))) float Bs[2][TK][TN + LDS_PAD];
  const long long M = a.counts[a.hop];
  // workgroup -> (tile, part of the contraction); the parts of a tile are n_tiles apart, so they keep its XCD
  const int id = (int)blockIdx.x % a.n_tiles, part_id = (int)blockIdx.x / a.n_tiles;
  const int xcd = id & 7, j = id >> 3;
  const int nt = j % a.n_tiles_n;
  const long long row0 = ((long long)(j / a.n_tiles_n) * 8 + xcd) * TM;
  const int col0 = nt * TN;
  if (row0 >= M) return;
  const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int K = a.K, N = a.N;
  const int kt_per_src = (K + TK - 1) / TK;
  // the slab loop is unrolled by two; with a single operand pair an odd slab count is rounded up
  // by one slab that lies wholly beyond K and therefore loads zeros
  const int n_kt = a.single ? (kt_per_src + 1) / 2 * 2 : 2 * kt_per_src;
  // this workgroup's slabs [kt_lo, kt_hi), in whole pairs (the host keeps split <= n_kt / 2)
  const int kt_lo = (int)((long long)(n_kt / 2) * part_id / a.split) * 2;
  const int kt_hi = (int)((long long)(n_kt / 2) * (part_id + 1) / a.split) * 2;

  // two accumulators (even / odd k pairs) so that consecutive matrix instructions are independent
  floatx16 acc, acc1;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    acc[r] = 0.f;
    acc1[r] = 0.f;
  }

  constexpr int kPer = TM * TK / kGemmThreads;  // floats of each operand per thread and slab
  auto load_slab = [&](int kt, float (&ra)[kPer], float (&rb)[kPer]) {
    const bool second = !a.single && kt >= kt_per_src;
    const float* A = (second || a.single) ? a.a_neigh : a.a_self;
    const float* W = (second || a.single) ? a.w_neigh : a.w_self;
    const int k0 = (second ? kt - kt_per_src : kt) * TK;
#pragma unroll
    for (int q = 0; q < kPer / VA; ++q) {
      const int e = tid + kGemmThreads * q;
      const int kc = e % (TK / VA), m = e / (TK / VA);
      const long long row = row0 + m;
      const int k = k0 + kc * VA;
      const bool ok = row < M && k < K;
      if (VA == 4) {
        const float4 v = ok ? *reinterpret_cast<const float4*>(A + row * K + k) : make_float4(0.f, 0.f, 0.f, 0.f);
        ra[4 * q] = v.x; ra[4 * q + 1] = v.y; ra[4 * q + 2] = v.z; ra[4 * q + 3] = v.w;
      } else if (VA == 2) {
        const float2 v = ok ? *reinterpret_cast<const float2*>(A + row * K + k) : make_float2(0.f, 0.f);
        ra[2 * q] = v.x; ra[2 * q + 1] = v.y;
      } else {
        ra[q] = ok ? A[row * K + k] : 0.f;
      }
    }
#pragma unroll
    for (int q = 0; q < kPer / VB; ++q) {
      const int e = tid + kGemmThreads * q;
      const int nc = e % (TN / VB), kk = e / (TN / VB);
      const int n = col0 + nc * VB;
      const bool ok = k0 + kk < K && n < N;
      if (VB == 4) {
        const float4 v = ok ? *reinterpret_cast<const float4*>(W + (long long)(k0 + kk) * N + n) : make_float4(0.f, 0.f, 0.f, 0.f);
        rb[4 * q] = v.x; rb[4 * q + 1] = v.y; rb[4 * q + 2] = v.z; rb[4 * q + 3] = v.w;
      } else {
        rb[q] = ok ? W[(long long)(k0 + kk) * N + n] : 0.f;
      }
    }
  };
  auto store_slab = [&](int buf, const float (&ra)[kPer], const float (&rb)[kPer]) {
#pragma unroll
    for (int q = 0; q < kPer / VA; ++q) {
      const int e = tid + kGemmThreads * q;
      const int kc = e % (TK / VA), m = e / (TK / VA);
#pragma unroll
      for (int v = 0; v < VA; ++v) As[buf][kc * VA + v][m] = ra[VA * q + v];
    }
#pragma unroll
    for (int q = 0; q < kPer / VB; ++q) {
      const int e = tid + kGemmThreads * q;
      const int nc = e % (TN / VB), kk = e / (TN / VB);
      if (VB == 4)
        *reinterpret_cast<float4*>(&Bs[buf][kk][nc * 4]) = make_float4(rb[4 * q], rb[4 * q + 1], rb[4 * q + 2], rb[4 * q + 3]);
      else
        Bs[buf][kk][nc] = rb[q];
    }
  };
  const int am = wm * 32 + (lane & 31), bn = wn * 32 + (lane & 31), kh = lane >> 5;
  auto compute = [&](int buf) {
#pragma unroll
    for (int kk = 0; kk < TK / 2; kk += 2) {
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(As[buf][2 * kk + kh][am], Bs[buf][2 * kk + kh][bn], acc, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(As[buf][2 * kk + 2 + kh][am], Bs[buf][2 * kk + 2 + kh][bn], acc1, 0, 0, 0);
    }
  };

  // Software pipeline over the (even number of) k-slabs: while slab kt is multiplied out of one
  // LDS buffer, slab kt+1 sits in registers on its way to the other buffer and the global loads
  // of slab kt+2 are already in flight, so a slab has two iterations to arrive.
  float ra0[kPer], rb0[kPer], ra1[kPer], rb1[kPer];
  load_slab(kt_lo, ra0, rb0);
  load_slab(kt_lo + 1, ra1, rb1);
  store_slab(0, ra0, rb0);
  __syncthreads();
  for (int kt = kt_lo; kt < kt_hi; kt += 2) {
    if (kt + 2 < kt_hi) load_slab(kt + 2, ra0, rb0);
    compute(0);
    store_slab(1, ra1, rb1);
    __syncthreads();
    if (kt + 3 < kt_hi) load_slab(kt + 3, ra1, rb1);
    compute(1);
    if (kt + 2 < kt_hi) store_slab(0, ra0, rb0);
    __syncthreads();
  }
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] += acc1[r];

  if (a.split > 1) {
    // partial sums go to this part's plane; k_split_reduce adds the planes in plane order
    const int col = col0 + bn;
    if (col < N) {
      float* plane = a.part + (size_t)part_id * a.part_rows * N;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const long long row = row0 + wm * 32 + 8 * (r >> 2) + 4 * kh + (r & 3);
        if (row < M) plane[row * N + col] = acc[r];
      }
    }
    return;
  }

  // accumulator layout of the 32x32 tile: register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4,
  // column l%32.
  const int col = col0 + bn;
  if (col < N) {
    const float b = a.bias[col];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const long long row = row0 + wm * 32 + 8 * (r >> 2) + 4 * kh + (r & 3);
      if (row < M) {
        float v = acc[r] + b;
        if (a.relu) v = v > 0.f ? v : 0.f;
        a.y[row * N + col] = v;
      }
    }
  }
}

// y = [relu](bias + sum over the planes, in plane order) for the rows in use
__global__ __launch_bounds__(256) void k_split_reduce(LinearArgs a) {
  const long long M = a.counts[a.hop];
  const long long total = M * a.N;
  const size_t plane = (size_t)a.part_rows * a.N;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
    float v = 0.f;
    for (int p = 0; p < a.split; ++p) v += a.part[p * plane + i];
    v += a.bias[i % a.N];
    if (a.relu) v = v > 0.f ? v : 0.f;
    a.y[i] = v;
  }
}

// ---- wide variant of the dense layer ----------------------------------------------------------
// Same product, for outputs whose width is a multiple of 128 and enough rows to matter.  One
// workgroup of eight wavefronts per compute unit (its LDS allotment admits no second one); a
// workgroup owns one 128-column tile and a contiguous share of the 32-row blocks, sized on the device
// from the row count, and walks its share in passes of up to six row blocks (192 x 128 outputs).
// Wave w multiplies columns 32*(w&3); the row blocks of a pass are split between w>>2 = 0 and 1, so
// the two wavefronts that share a SIMD also share the B fragment values and differ in A.
//
// Data movement is what limits this layer (a 64x64 tile moves 8 KB from L2 per 131 kflop and every
// vector-ALU instruction displaces a matrix instruction), so here
//  * operands go global -> LDS directly (16 bytes per lane, no registers, no address arithmetic on
//    the vector ALU: a scalar base per k-slab plus a constant lane offset);
//  * three stages of 16-deep k-slabs ring through LDS; slab i+3 is requested while slab i is
//    multiplied, and the fragments of slab i+1 are read into a second register set meanwhile;
//  * A is stored [row][4 chunks of 4 k] with the chunk index xor-ed by row bits, so a 16-byte
//    fragment read (four consecutive k of one row = four matrix instructions) is conflict free;
//    the contraction index is permuted consistently on both operands: matrix step (t, j) takes
//    k = 8t + j from lanes 0..31 and k = 8t + 4 + j from lanes 32..63;
//  * the loop is unrolled over (stage x register set) = 6 so that all LDS offsets are immediates;
//  * loads, fragment reads and matrix instructions are interleaved in a fixed order
//    (sched_barrier) so that the non-matrix issue slots hide behind the 64-cycle matrix ops.
// Fragment reads are inline assembly: the compiler would otherwise order every LDS read behind all
// outstanding global->LDS loads.  The columns K % 16 left over per operand go through registers
// with masks after the pipelined loop.
typedef float float2v __attribute__((ext_vector_type(2)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) const void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;
// A 16-byte load through a pointer that is known to be global memory.  An address that went through an integer (a
// shuffle, a note in LDS) has lost its address space; loaded through a generic pointer it would count against the
// LDS counter as well as the memory counter, and every wait for an LDS read would wait for it too.
typedef __attribute__((address_space(1))) const float4v* gf4ptr_t;
typedef __attribute__((address_space(1))) const float* gfptr_t;
__device__ __forceinline__ float4v load_global_f4(const float* p) { return *(gf4ptr_t)(p); }

constexpr long long kWideMinRows = 16384;  // below this capacity the 64x64 kernel (with its split contraction) fills the chip better
constexpr int kWideMinWidth = 192;  // narrower inputs spend the kernel in its pipeline fill and drain (measured cross-over with the 64x64 kernel)
constexpr int kWideThreads = 512, kWideCols = 128, kWideStages = 3, kWideMaxBlocks = 6;
constexpr int kWideABytes = kWideMaxBlocks * 32 * 64;           // 192 rows x 16 k x 4 B
constexpr int kWideBBytes = TK * kWideCols * 4;                 // 16 k x 128 columns x 4 B
constexpr int kWideStageBytes = kWideABytes + kWideBBytes;      // 20 KB
constexpr int kWideLdsBytes = 84 * 1024;                        // > half of the 160 KB: one workgroup per CU
static_assert(kWideStages * kWideStageBytes <= 65536, "LDS offsets must fit the 16-bit immediates");
static_assert(kWideStages * kWideStageBytes <= kWideLdsBytes, "stages must fit the allocation");

struct FragW {
  float4v a[3][2];  // [row block][t]: four consecutive k of this lane's row
  float2v b[4];     // steps (t=0: j=0,1), (0: 2,3), (1: 0,1), (1: 2,3) of this lane's column
};

#define DCI_DS_READ_A2(x0, x1, a0_, a1_, OFF)                                     \
  asm volatile("ds_read_b128 %0, %2 offset:%4\n\tds_read_b128 %1, %3 offset:%4"  \
               : "=&v"(x0), "=&v"(x1)                                             \
               : "v"(a0_), "v"(a1_), "n"(OFF)                                     \
               : "memory")
#define DCI_DS_READ_B4(y0, y1, y2, y3, b_, U0)                                                                       \
  asm volatile("ds_read2st64_b32 %0, %4 offset0:%5 offset1:%6\n\tds_read2st64_b32 %1, %4 offset0:%7 offset1:%8\n\t" \
               "ds_read2st64_b32 %2, %4 offset0:%9 offset1:%10\n\tds_read2st64_b32 %3, %4 offset0:%11 offset1:%12"  \
               : "=&v"(y0), "=&v"(y1), "=&v"(y2), "=&v"(y3)                                                          \
               : "v"(b_), "n"((U0) + 0), "n"((U0) + 2), "n"((U0) + 4), "n"((U0) + 6), "n"((U0) + 16),                \
                 "n"((U0) + 18), "n"((U0) + 20), "n"((U0) + 22)                                                      \
               : "memory")
// waits until at most VM of this wave's global->LDS loads are outstanding and all its LDS reads have
// returned; the second statement ties every fragment register to the wait
#define DCI_WAIT_FRAG(f, VM)                                                                                         \
  do {                                                                                                               \
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(VM) : "memory");                                             \
    asm volatile("" : "+v"(f.a[0][0]), "+v"(f.a[0][1]), "+v"(f.a[1][0]), "+v"(f.a[1][1]), "+v"(f.a[2][0]),           \
                      "+v"(f.a[2][1]), "+v"(f.b[0]), "+v"(f.b[1]), "+v"(f.b[2]), "+v"(f.b[3])::"memory");            \
  } while (0)

// kInputLayer only gives the first layer's launches a kernel name of their own in traces; the code is the same.
template <bool kInputLayer>
__global__ __launch_bounds__(kWideThreads, 1) void k_sage_linear_wide(LinearArgs a, int g_n) {
  constexpr int NS = kWideStages, ST = kWideStageBytes, LPW = 3;  // LPW: global->LDS loads per wave and slab
  __shared__ __attribute__((aligned(1024))) char lds[kWideLdsBytes];
  const long long M = a.counts[a.hop];
  const int id = (int)blockIdx.x;
  const int xcd = id & 7, jj = id >> 3;
  const int nt = jj % a.n_tiles_n;
  const int slot = (jj / a.n_tiles_n) * 8 + xcd;   // the column tiles of one row share run on one XCD
  if (slot >= g_n) return;
  const long long n_rb = (M + 31) / 32;
  const long long chunk = (n_rb + g_n - 1) / g_n;
  const long long rb_begin = (long long)slot * chunk;
  long long rb_end = rb_begin + chunk;
  if (rb_end > n_rb) rb_end = n_rb;
  if (rb_begin >= rb_end) return;
  const int col0 = nt * kWideCols;
  const int tid = (int)threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wc = wave & 3, wr = wave >> 2;
  const int K = a.K, N = a.N;
  const int Sf = K / TK;                   // full slabs per operand
  const int n = a.single ? Sf : 2 * Sf;    // slabs of the pipelined loop
  const int k_tail = K - Sf * TK;
  const int c_a = (lane & 3) ^ ((lane >> 4) & 3);
  const int h = lane >> 5, ll = lane & 31;
  const unsigned lds0 = (unsigned)(size_t)(lptr_t)lds;
  const unsigned lb0 = lds0 + 4 * h * kWideCols * 4 + (((wc * 32 + ll) ^ (32 * h)) * 4);
  const int krB = 2 * wave + (lane >> 5);  // this lane's k row of the B slab
  const unsigned voffB = (unsigned)((krB * N + (((lane & 31) ^ (8 * ((krB >> 2) & 1))) * 4)) * 4);
  const float* pW0 = (a.single ? a.w_neigh : a.w_self) + col0;
  const float* pW1 = a.w_neigh + col0;
  const int col = col0 + wc * 32 + ll;
  const float bias = a.bias[col];
  const int ldsA1 = (wave + 8 > 2 * kWideMaxBlocks - 1 ? 2 * kWideMaxBlocks - 1 : wave + 8) * 1024;

  const int cnt = (int)(rb_end - rb_begin);
  const int n_pass = (cnt + kWideMaxBlocks - 1) / kWideMaxBlocks;
  const int per = (cnt + n_pass - 1) / n_pass;
  for (long long prb = rb_begin; prb < rb_end; prb += per) {
    const int r_eff = (int)((rb_end - prb) < per ? (rb_end - prb) : per);  // 1..6 row blocks in this pass
    const int rw0 = (r_eff + 1) / 2;
    const int rw = wr == 0 ? rw0 : r_eff - rw0;                             // row blocks of this wave (0..3)
    const long long row0 = prb * 32;
    // the 16-row groups this wave fetches (wave and wave + 8, the latter clamped: four waves repeat
    // group 11); rows past M repeat row M-1 and are never stored
    unsigned voffA[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      int i = wave + 8 * q;
      if (i > 2 * kWideMaxBlocks - 1) i = 2 * kWideMaxBlocks - 1;
      long long r = row0 + 16 * i + (lane >> 2);
      if (r > M - 1) r = M - 1;
      voffA[q] = (unsigned)(((r - row0) * K + c_a * 4) * 4);
    }
    const float* pA0 = (a.single ? a.a_neigh : a.a_self) + row0 * K;
    const float* pA1 = a.a_neigh + row0 * K;
    const unsigned la0 = lds0 + (wr * rw0 * 32 + ll) * 64 + ((h ^ ((ll >> 2) & 3)) * 16);
    const unsigned la1 = la0 ^ 32u;
    floatx16 acc[3];
#pragma unroll
    for (int rb = 0; rb < 3; ++rb)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[rb][r] = 0.f;

#define DCI_SLAB_PTRS(s_)                                                                            \
  const bool second_ = (s_) >= Sf && !a.single;                                                      \
  const int ks_ = second_ ? (s_) - Sf : (s_);                                                        \
  const char* ga_ = reinterpret_cast<const char*>((second_ ? pA1 : pA0) + ks_ * TK);                 \
  const char* gw_ = reinterpret_cast<const char*>((second_ ? pW1 : pW0) + (size_t)ks_ * TK * N)
#define DCI_LOAD_A0(STG) \
  __builtin_amdgcn_global_load_lds((gptr_t)(ga_ + voffA[0]), (lptr_t)(lds + (STG)*ST + wave * 1024), 16, 0, 0)
#define DCI_LOAD_A1(STG) \
  __builtin_amdgcn_global_load_lds((gptr_t)(ga_ + voffA[1]), (lptr_t)(lds + (STG)*ST + ldsA1), 16, 0, 0)
#define DCI_LOAD_B(STG) \
  __builtin_amdgcn_global_load_lds((gptr_t)(gw_ + voffB), (lptr_t)(lds + (STG)*ST + kWideABytes + wave * 1024), 16, 0, 0)
#define DCI_ISSUE(s_, STG) \
  do {                     \
    DCI_SLAB_PTRS(s_);     \
    DCI_LOAD_A0(STG);      \
    DCI_LOAD_A1(STG);      \
    DCI_LOAD_B(STG);       \
  } while (0)
#define DCI_READ(f, STG)                                                                  \
  do {                                                                                    \
    DCI_DS_READ_A2(f.a[0][0], f.a[0][1], la0, la1, (STG)*ST + 0 * 2048);                  \
    DCI_DS_READ_A2(f.a[1][0], f.a[1][1], la0, la1, (STG)*ST + 1 * 2048);                  \
    DCI_DS_READ_A2(f.a[2][0], f.a[2][1], la0, la1, (STG)*ST + 2 * 2048);                  \
    DCI_DS_READ_B4(f.b[0], f.b[1], f.b[2], f.b[3], lb0, ((STG)*ST + kWideABytes) / 256);  \
  } while (0)
// matrix step (t_, j_) of every row block of this wave
#define DCI_MFMA_G(f, t_, j_)                                                                                          \
  do {                                                                                                                 \
    const float bv_ = ((j_) & 1) ? f.b[2 * (t_) + ((j_) >> 1)].y : f.b[2 * (t_) + ((j_) >> 1)].x;                      \
    _Pragma("unroll") for (int rb_ = 0; rb_ < 3; ++rb_) {                                                              \
      const float av_ = (j_) == 0 ? f.a[rb_][t_].x : (j_) == 1 ? f.a[rb_][t_].y : (j_) == 2 ? f.a[rb_][t_].z : f.a[rb_][t_].w; \
      if (rb_ < rw) acc[rb_] = __builtin_amdgcn_mfma_f32_32x32x2f32(av_, bv_, acc[rb_], 0, 0, 0);                      \
    }                                                                                                                  \
    __builtin_amdgcn_sched_barrier(0);                                                                                 \
  } while (0)
#define DCI_MFMA_SLAB(f)                                       \
  do {                                                         \
    __builtin_amdgcn_sched_barrier(0);                         \
    DCI_MFMA_G(f, 0, 0); DCI_MFMA_G(f, 0, 1); DCI_MFMA_G(f, 0, 2); DCI_MFMA_G(f, 0, 3); \
    DCI_MFMA_G(f, 1, 0); DCI_MFMA_G(f, 1, 1); DCI_MFMA_G(f, 1, 2); DCI_MFMA_G(f, 1, 3); \
  } while (0)
// steady state: slab idx is multiplied from FC while slab idx+3 is requested into the stage it
// leaves (U % 3) and the fragments of slab idx+1 are read into FN
#define DCI_STEP(FC, FN, idx, U)                                                      \
  do {                                                                                \
    DCI_WAIT_FRAG(FC, LPW * (NS - 2));                                                \
    __builtin_amdgcn_s_barrier();                                                     \
    const char* ga_ = ga_run;                                                         \
    const char* gw_ = gw_run;                                                         \
    __builtin_amdgcn_sched_barrier(0);                                                \
    DCI_MFMA_G(FC, 0, 0);                                                             \
    DCI_LOAD_A0((U) % 3);                                                             \
    __builtin_amdgcn_sched_barrier(0);                                                \
    DCI_MFMA_G(FC, 0, 1);                                                             \
    DCI_LOAD_A1((U) % 3);                                                             \
    __builtin_amdgcn_sched_barrier(0);                                                \
    DCI_MFMA_G(FC, 0, 2);                                                             \
    DCI_LOAD_B((U) % 3);                                                              \
    __builtin_amdgcn_sched_barrier(0);                                                \
    DCI_MFMA_G(FC, 0, 3);                                                             \
    DCI_DS_READ_A2(FN.a[0][0], FN.a[0][1], la0, la1, (((U) + 1) % 3) * ST + 0 * 2048); \
    __builtin_amdgcn_sched_barrier(0);                                                \
    DCI_MFMA_G(FC, 1, 0);                                                             \
    DCI_DS_READ_A2(FN.a[1][0], FN.a[1][1], la0, la1, (((U) + 1) % 3) * ST + 1 * 2048); \
    __builtin_amdgcn_sched_barrier(0);                                                \
    DCI_MFMA_G(FC, 1, 1);                                                             \
    DCI_DS_READ_A2(FN.a[2][0], FN.a[2][1], la0, la1, (((U) + 1) % 3) * ST + 2 * 2048); \
    __builtin_amdgcn_sched_barrier(0);                                                \
    DCI_MFMA_G(FC, 1, 2);                                                             \
    DCI_DS_READ_B4(FN.b[0], FN.b[1], FN.b[2], FN.b[3], lb0, ((((U) + 1) % 3) * ST + kWideABytes) / 256); \
    __builtin_amdgcn_sched_barrier(0);                                                \
    DCI_MFMA_G(FC, 1, 3);                                                             \
    /* running operand pointers: one slab on; at the end of the first operand over to the second */ \
    ga_run += TK * 4;                                                                 \
    gw_run += (size_t)TK * N * 4;                                                     \
    if (++ks_run == Sf) {                                                             \
      ks_run = 0;                                                                     \
      ga_run = reinterpret_cast<const char*>(pA1);                                    \
      gw_run = reinterpret_cast<const char*>(pW1);                                    \
    }                                                                                 \
  } while (0)

    if (n > 0) {
      FragW fa, fb;
      if (n > 0) DCI_ISSUE(0, 0);
      if (n > 1) DCI_ISSUE(1, 1);
      if (n > 2) DCI_ISSUE(2, 2);
      if (n >= NS) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LPW * (NS - 1)) : "memory");
      else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __builtin_amdgcn_s_barrier();
      DCI_READ(fa, 0);
      // the slab the steady-state loop requests next (slab NS first): operand, slab within it, addresses
      const bool run_second = NS >= Sf && !a.single;
      int ks_run = run_second ? NS - Sf : NS;
      const char* ga_run = reinterpret_cast<const char*>((run_second ? pA1 : pA0) + ks_run * TK);
      const char* gw_run = reinterpret_cast<const char*>((run_second ? pW1 : pW0) + (size_t)ks_run * TK * N);
      int i = 0;
      for (; i + 5 + NS < n; i += 6) {  // i % 6 == 0: slab i+u sits in stage u % 3, all indices are valid slabs
        DCI_STEP(fa, fb, i, 0);
        DCI_STEP(fb, fa, i + 1, 1);
        DCI_STEP(fa, fb, i + 2, 2);
        DCI_STEP(fb, fa, i + 3, 3);
        DCI_STEP(fa, fb, i + 4, 4);
        DCI_STEP(fb, fa, i + 5, 5);
      }
      // drain (at most eight slabs): stage chosen at run time, every wait is for everything
      for (; i + 1 < n; ++i) {
        DCI_WAIT_FRAG(fa, 0);
        __builtin_amdgcn_s_barrier();
        if (i + NS < n) {
          const int st_ = i % NS;
          if (st_ == 0) DCI_ISSUE(i + NS, 0);
          else if (st_ == 1) DCI_ISSUE(i + NS, 1);
          else DCI_ISSUE(i + NS, 2);
        }
        const int sn_ = (i + 1) % NS;
        if (sn_ == 0) DCI_READ(fb, 0);
        else if (sn_ == 1) DCI_READ(fb, 1);
        else DCI_READ(fb, 2);
        DCI_MFMA_SLAB(fa);
        fa = fb;
      }
      DCI_WAIT_FRAG(fa, 0);
      DCI_MFMA_SLAB(fa);
    }
    if (k_tail > 0) {
      // the last k_tail columns of each operand: masked loads through registers into stage 0
      const int n_ops = a.single ? 1 : 2;
      for (int o = 0; o < n_ops; ++o) {
        const float* A = (o == 1 ? pA1 : pA0) + Sf * TK;
        const float* W = (o == 1 ? pW1 : pW0) + (size_t)Sf * TK * N;
        float4 va[2];
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          float v[4];
#pragma unroll
          for (int e = 0; e < 4; ++e)
            v[e] = (Sf * TK + 4 * c_a + e < K)
                       ? *reinterpret_cast<const float*>(reinterpret_cast<const char*>(A + e) + voffA[q])
                       : 0.f;
          va[q] = make_float4(v[0], v[1], v[2], v[3]);
        }
        const float4 w = (Sf * TK + krB < K) ? *reinterpret_cast<const float4*>(reinterpret_cast<const char*>(W) + voffB)
                                             : make_float4(0.f, 0.f, 0.f, 0.f);
        __syncthreads();  // every wave has its fragments of the slab that used stage 0 last
        *reinterpret_cast<float4*>(lds + wave * 1024 + lane * 16) = va[0];
        *reinterpret_cast<float4*>(lds + ldsA1 + lane * 16) = va[1];
        *reinterpret_cast<float4*>(lds + kWideABytes + wave * 1024 + lane * 16) = w;
        __syncthreads();
        FragW f;
        DCI_READ(f, 0);
        DCI_WAIT_FRAG(f, 0);
        DCI_MFMA_SLAB(f);
      }
    }
#pragma unroll
    for (int rb = 0; rb < 3; ++rb) {
      if (rb < rw) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const long long row = row0 + (wr * rw0 + rb) * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
          if (row < M) {
            float v = acc[rb][r] + bias;
            if (a.relu) v = v > 0.f ? v : 0.f;
            a.y[row * N + col] = v;
          }
        }
      }
    }
    __syncthreads();  // the next pass refills the stages
  }
#undef DCI_SLAB_PTRS
#undef DCI_LOAD_A0
#undef DCI_LOAD_A1
#undef DCI_LOAD_B
#undef DCI_ISSUE
#undef DCI_READ
#undef DCI_MFMA_G
#undef DCI_MFMA_SLAB
#undef DCI_STEP
}

// ---- 64x64 tiles fed by global->LDS loads ---------------------------------------------------
// The tile kernel's shape (one 32x32 tile per wavefront, four wavefronts, XCD-aware order) with the
// wide kernel's data path: 16-byte global->LDS loads (two per wave and slab), three stages of
// 16-deep slabs, inline-assembly fragment reads with immediate offsets, no vector-ALU work in the
// steady-state loop.  Its slab costs about 0.4 us where the register path needs 0.6-0.8 us, which
// is what counts for layers of a few thousand rows (every workgroup walks the whole contraction)
// and for narrow inputs; at tens of thousands of rows and wide inputs it has no edge over the tile
// kernel and loses to the wide one.  Needs an output width that is a multiple of 64, an even
// input width, 8-byte aligned rows and 16-byte aligned weights.
struct FragD {
  float4v a0, a1;           // t = 0, 1: four consecutive k of this lane's row
  float2v b0, b1, b2, b3;   // steps (0: 0,1), (0: 2,3), (1: 0,1), (1: 2,3) of this lane's column
};
constexpr int kDmaStages = 3, kDmaStageBytes = (TM * TK + TK * TN) * 4;  // 8 KB
static_assert(TM == 64 && TN == 64 && TK == 16, "the layout below is written for 64x64x16");

#define DCI_D_READ(f, STG)                                                                                            \
  asm volatile("ds_read_b128 %0, %6 offset:%9\n\tds_read_b128 %1, %7 offset:%9\n\t"                                  \
               "ds_read2st64_b32 %2, %8 offset0:%10 offset1:%11\n\tds_read2st64_b32 %3, %8 offset0:%12 offset1:%13\n\t" \
               "ds_read2st64_b32 %4, %8 offset0:%14 offset1:%15\n\tds_read2st64_b32 %5, %8 offset0:%16 offset1:%17"  \
               : "=&v"(f.a0), "=&v"(f.a1), "=&v"(f.b0), "=&v"(f.b1), "=&v"(f.b2), "=&v"(f.b3)                         \
               : "v"(la0), "v"(la1), "v"(lb0), "n"((STG)*kDmaStageBytes), "n"((STG)*32 + 16), "n"((STG)*32 + 17),     \
                 "n"((STG)*32 + 18), "n"((STG)*32 + 19), "n"((STG)*32 + 24), "n"((STG)*32 + 25), "n"((STG)*32 + 26),  \
                 "n"((STG)*32 + 27)                                                                                   \
               : "memory")
#define DCI_D_WAIT(f, VM)                                                                                             \
  do {                                                                                                                \
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(VM) : "memory");                                              \
    asm volatile("" : "+v"(f.a0), "+v"(f.a1), "+v"(f.b0), "+v"(f.b1), "+v"(f.b2), "+v"(f.b3)::"memory");              \
  } while (0)

__global__ __launch_bounds__(kGemmThreads) void k_sage_linear_dma(LinearArgs a) {
  constexpr int NS = kDmaStages, ST = kDmaStageBytes, A_BYTES = TM * TK * 4, LPW = 2;
  __shared__ __attribute__((aligned(1024))) char lds[NS * ST];
  const long long M = a.counts[a.hop];
  const int id = (int)blockIdx.x;
  const int xcd = id & 7, jj = id >> 3;
  const int nt = jj % a.n_tiles_n;
  const long long row0 = ((long long)(jj / a.n_tiles_n) * 8 + xcd) * TM;
  const int col0 = nt * TN;
  if (row0 >= M) return;
  const int tid = (int)threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int K = a.K, N = a.N;
  const int Sf = K / TK;
  const int n = a.single ? Sf : 2 * Sf;
  const int k_tail = K - Sf * TK;
  // this wave's share of a slab: rows 16*wave .. +15 of A (lane -> row, chunk of four k; chunk position
  // xor-ed with row bits), k rows 4*wave .. +3 of B (column halves swapped in every second group of four rows)
  const int c_a = (lane & 3) ^ ((lane >> 4) & 3);
  long long r_l = row0 + 16 * wave + (lane >> 2);
  if (r_l > M - 1) r_l = M - 1;
  const unsigned voffA = (unsigned)(((r_l - row0) * K + c_a * 4) * 4);
  const int krB = 4 * wave + (lane >> 4);
  const unsigned voffB = (unsigned)((krB * N + (((lane & 15) ^ (8 * (wave & 1))) * 4)) * 4);
  const float* pA0 = (a.single ? a.a_neigh : a.a_self) + row0 * K;
  const float* pA1 = a.a_neigh + row0 * K;
  const float* pW0 = (a.single ? a.w_neigh : a.w_self) + col0;
  const float* pW1 = a.w_neigh + col0;
  char* const ldsw = lds + 1024 * wave;
  const int wm = wave >> 1, wn = wave & 1;
  const int h = lane >> 5, ll = lane & 31;
  const int am = wm * 32 + ll;
  const unsigned lds0 = (unsigned)(size_t)(lptr_t)lds;
  const unsigned la0 = lds0 + am * 64 + ((h ^ ((am >> 2) & 3)) * 16);
  const unsigned la1 = la0 ^ 32u;
  const unsigned lb0 = lds0 + 4 * h * TN * 4 + (((wn * 32 + ll) ^ (32 * h)) * 4);  // the B region offset sits in the immediates
  floatx16 acc0, acc1;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    acc0[r] = 0.f;
    acc1[r] = 0.f;
  }

#define DCI_D_ISSUE(s_, STG)                                                                                  \
  do {                                                                                                        \
    const bool second_ = (s_) >= Sf && !a.single;                                                             \
    const int ks_ = second_ ? (s_) - Sf : (s_);                                                               \
    const char* ga_ = reinterpret_cast<const char*>((second_ ? pA1 : pA0) + ks_ * TK);                        \
    const char* gw_ = reinterpret_cast<const char*>((second_ ? pW1 : pW0) + (size_t)ks_ * TK * N);            \
    __builtin_amdgcn_global_load_lds((gptr_t)(ga_ + voffA), (lptr_t)(ldsw + (STG)*ST), 16, 0, 0);             \
    __builtin_amdgcn_global_load_lds((gptr_t)(gw_ + voffB), (lptr_t)(ldsw + (STG)*ST + A_BYTES), 16, 0, 0);   \
  } while (0)
#define DCI_D_MFMA(f)                                                              \
  do {                                                                             \
    __builtin_amdgcn_sched_barrier(0);                                             \
    acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a0.x, f.b0.x, acc0, 0, 0, 0);    \
    acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a0.y, f.b0.y, acc1, 0, 0, 0);    \
    acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a0.z, f.b1.x, acc0, 0, 0, 0);    \
    acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a0.w, f.b1.y, acc1, 0, 0, 0);    \
    acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a1.x, f.b2.x, acc0, 0, 0, 0);    \
    acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a1.y, f.b2.y, acc1, 0, 0, 0);    \
    acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a1.z, f.b3.x, acc0, 0, 0, 0);    \
    acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a1.w, f.b3.y, acc1, 0, 0, 0);    \
    __builtin_amdgcn_sched_barrier(0);                                             \
  } while (0)
#define DCI_D_STEP(FC, FN, idx, U)     \
  do {                                 \
    DCI_D_WAIT(FC, LPW * (NS - 2));    \
    __builtin_amdgcn_s_barrier();      \
    DCI_D_ISSUE((idx) + NS, (U) % 3);  \
    DCI_D_READ(FN, ((U) + 1) % 3);     \
    DCI_D_MFMA(FC);                    \
  } while (0)

  if (n > 0) {
    FragD fa, fb;
    if (n > 0) DCI_D_ISSUE(0, 0);
    if (n > 1) DCI_D_ISSUE(1, 1);
    if (n > 2) DCI_D_ISSUE(2, 2);
    if (n >= NS) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LPW * (NS - 1)) : "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    DCI_D_READ(fa, 0);
    int i = 0;
    for (; i + 5 + NS < n; i += 6) {  // i % 6 == 0: slab i+u sits in stage u % 3, all indices are valid slabs
      DCI_D_STEP(fa, fb, i, 0);
      DCI_D_STEP(fb, fa, i + 1, 1);
      DCI_D_STEP(fa, fb, i + 2, 2);
      DCI_D_STEP(fb, fa, i + 3, 3);
      DCI_D_STEP(fa, fb, i + 4, 4);
      DCI_D_STEP(fb, fa, i + 5, 5);
    }
    for (; i + 1 < n; ++i) {  // drain: stage chosen at run time, every wait is for everything
      DCI_D_WAIT(fa, 0);
      __builtin_amdgcn_s_barrier();
      if (i + NS < n) {
        const int st_ = i % NS;
        if (st_ == 0) DCI_D_ISSUE(i + NS, 0);
        else if (st_ == 1) DCI_D_ISSUE(i + NS, 1);
        else DCI_D_ISSUE(i + NS, 2);
      }
      const int sn_ = (i + 1) % NS;
      if (sn_ == 0) DCI_D_READ(fb, 0);
      else if (sn_ == 1) DCI_D_READ(fb, 1);
      else DCI_D_READ(fb, 2);
      DCI_D_MFMA(fa);
      fa = fb;
    }
    DCI_D_WAIT(fa, 0);
    DCI_D_MFMA(fa);
  }
  if (k_tail > 0) {
    // the last k_tail columns of each operand: masked loads through registers into stage 0
    const int n_ops = a.single ? 1 : 2;
    for (int o = 0; o < n_ops; ++o) {
      const float* A = (o == 1 ? pA1 : pA0) + Sf * TK;
      const float* W = (o == 1 ? pW1 : pW0) + (size_t)Sf * TK * N;
      float v[4];
#pragma unroll
      for (int e = 0; e < 4; ++e)
        v[e] = (Sf * TK + 4 * c_a + e < K)
                   ? *reinterpret_cast<const float*>(reinterpret_cast<const char*>(A + e) + voffA)
                   : 0.f;
      const float4 w = (Sf * TK + krB < K) ? *reinterpret_cast<const float4*>(reinterpret_cast<const char*>(W) + voffB)
                                           : make_float4(0.f, 0.f, 0.f, 0.f);
      __syncthreads();  // every wave has its fragments of the slab that used stage 0 last
      *reinterpret_cast<float4*>(ldsw + lane * 16) = make_float4(v[0], v[1], v[2], v[3]);
      *reinterpret_cast<float4*>(ldsw + A_BYTES + lane * 16) = w;
      __syncthreads();
      FragD f;
      DCI_D_READ(f, 0);
      DCI_D_WAIT(f, 0);
      DCI_D_MFMA(f);
    }
  }
#pragma unroll
  for (int r = 0; r < 16; ++r) acc0[r] += acc1[r];
  const int col = col0 + wn * 32 + ll;
  const float b = a.bias[col];
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const long long row = row0 + wm * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
    if (row < M) {
      float v = acc0[r] + b;
      if (a.relu) v = v > 0.f ? v : 0.f;
      a.y[row * N + col] = v;
    }
  }
#undef DCI_D_ISSUE
#undef DCI_D_MFMA
#undef DCI_D_STEP
}

// ---- weights resident in registers -------------------------------------------------------------
// For layers whose whole contraction is at most 256 long (two operands of up to 128 columns each, or a
// single one of up to 256) and whose output width is a multiple of 256.  With so short a contraction a
// tiled kernel spends its time filling and draining its pipeline and re-reading the weights for every
// tile; here each of the eight wavefronts of a workgroup owns 32 output columns and keeps its share of
// the weights (contraction length x 32 values = up to 128 registers per lane) for the whole launch.
// A workgroup (one per compute unit) walks 32-row blocks of the activations: a block's rows (both
// operands side by side, at most 32 KB) arrive in LDS by 16-byte global->LDS loads two blocks ahead
// (three buffers), every wavefront reads the whole block from LDS (16-byte fragment reads, same
// xor-swizzled [slab][row][4 chunks] layout as the other kernels) and runs the contraction as one chain
// of up to 128 matrix instructions into its 32x32 accumulator; the finished block is stored while the
// next one is multiplied (two accumulator sets).  One barrier per block.
// Needs: input width a multiple of 4, 16-byte aligned activation rows.
constexpr int kResThreads = 512, kResCols = 256, kResMaxSlabs = 16, kResBufs = 3;
constexpr int kResTileBytes = kResMaxSlabs * 32 * 64;  // 32 rows x 256 k x 4 B
constexpr long long kResMinRows = 98304;               // by capacity; batches fill a quarter of it or so, and below about five row blocks per compute unit the start-up (every workgroup fetches all the weights) outweighs the gain

struct FragR {
  float4v a0, a1;  // t = 0, 1: four consecutive k of this lane's row
};
#define DCI_R_READ(f, OFF)                                                        \
  asm volatile("ds_read_b128 %0, %2 offset:%4\n\tds_read_b128 %1, %3 offset:%4"  \
               : "=&v"(f.a0), "=&v"(f.a1)                                         \
               : "v"(la0), "v"(la1), "n"(OFF)                                     \
               : "memory")
#define DCI_R_WAIT(f, LG)                                                \
  do {                                                                   \
    asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(LG) : "memory");          \
    asm volatile("" : "+v"(f.a0), "+v"(f.a1)::"memory");                 \
  } while (0)
// slab S_ of the block: its fragments are in FC; the next slab's are requested into FN meanwhile.  NS (the
// kernel's slab count) is a compile-time constant, so the conditions fold and the block is straight-line code.
#define DCI_R_SLAB(S_, FC, FN, AC)                                                               \
  if ((S_) < NS) {                                                                               \
    DCI_R_WAIT(FC, 0); /* asked for a slab ago; a wait for everything does not depend on what else is counted */ \
    if ((S_) + 1 < NS) DCI_R_READ(FN, (((S_) + 1) % kResMaxSlabs) * 2048);                       \
    __builtin_amdgcn_sched_barrier(0);                                                           \
    AC = __builtin_amdgcn_mfma_f32_32x32x2f32(FC.a0.x, breg[8 * (S_) + 0], AC, 0, 0, 0);         \
    AC = __builtin_amdgcn_mfma_f32_32x32x2f32(FC.a0.y, breg[8 * (S_) + 1], AC, 0, 0, 0);         \
    AC = __builtin_amdgcn_mfma_f32_32x32x2f32(FC.a0.z, breg[8 * (S_) + 2], AC, 0, 0, 0);         \
    AC = __builtin_amdgcn_mfma_f32_32x32x2f32(FC.a0.w, breg[8 * (S_) + 3], AC, 0, 0, 0);         \
    AC = __builtin_amdgcn_mfma_f32_32x32x2f32(FC.a1.x, breg[8 * (S_) + 4], AC, 0, 0, 0);         \
    AC = __builtin_amdgcn_mfma_f32_32x32x2f32(FC.a1.y, breg[8 * (S_) + 5], AC, 0, 0, 0);         \
    AC = __builtin_amdgcn_mfma_f32_32x32x2f32(FC.a1.z, breg[8 * (S_) + 6], AC, 0, 0, 0);         \
    AC = __builtin_amdgcn_mfma_f32_32x32x2f32(FC.a1.w, breg[8 * (S_) + 7], AC, 0, 0, 0);         \
    __builtin_amdgcn_sched_barrier(0);                                                           \
  }

// NS: slabs of 16 the kernel multiplies, at least ceil(contraction length / 16); the weights and the LDS
// chunks beyond the real length are zero, so a larger NS only costs time.
template <int NS>
__global__ __launch_bounds__(kResThreads, 1) void k_sage_linear_res(LinearArgs a, int g_n) {
  static_assert(NS >= 1 && NS <= kResMaxSlabs, "slab count");
  __shared__ __attribute__((aligned(1024))) char lds[kResBufs * kResTileBytes];
  const long long M = a.counts[a.hop];
  const int id = (int)blockIdx.x;
  const int nt = id % a.n_tiles_n, slot = id / a.n_tiles_n;  // column tile, share of the row blocks
  const long long n_rb = (M + 31) / 32;
  if (slot >= n_rb) return;
  const int n_my = (int)((n_rb - slot + g_n - 1) / g_n);  // blocks slot, slot + g_n, ...
  const int tid = (int)threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int h = lane >> 5, ll = lane & 31;
  const int K = a.K, N = a.N;
  // The contraction runs over chunks of four k: first the chunks of the first operand, padded with a zero chunk
  // to an even count, then those of the second operand likewise (so a pair of chunks - what one matrix step
  // takes, one chunk per half of the wavefront - never straddles the operands), then zero chunks up to 4 NS.
  const int n_ops = a.single ? 1 : 2;
  const int kc_op = K / 4;                 // chunks of an operand that hold data
  const int kpc = (kc_op + 1) & ~1;        // chunks per operand in the padded sequence
  const float* A0 = a.single ? a.a_neigh : a.a_self;
  const float* W0 = a.single ? a.w_neigh : a.w_self;

  // Padding chunks are never loaded: they stay zero.
  if (n_ops * kc_op != 4 * NS)
    for (int i = tid; i < kResBufs * kResTileBytes / 16; i += kResThreads)
      reinterpret_cast<float4*>(lds)[i] = make_float4(0.f, 0.f, 0.f, 0.f);

  const int col = nt * kResCols + wave * 32 + ll;  // this lane's output column
  const float bias = a.bias[col];

  // Loads of a block: 2 per slab (16 rows each), numbered L = 2 slab + half; this wavefront issues
  // L = wave, wave + 8, wave + 16, wave + 24.  Lane -> row 16 half + lane / 4, chunk (lane & 3) xor-ed with row bits.
  const int rl = 16 * (wave & 1) + (lane >> 2);
  const int c_a = (lane & 3) ^ ((lane >> 4) & 3);
  const float* pb[4];
  bool valid[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = 4 * ((wave + 8 * i) >> 1) + c_a;  // this lane's chunk in the padded sequence
    const int op = c >= kpc ? 1 : 0;
    const int kc = c - op * kpc;
    valid[i] = op < n_ops && kc < kc_op;
    pb[i] = (op ? a.a_neigh : A0) + 4 * kc;
  }
  auto issue = [&](int it_, int buf_) {
    long long r = ((long long)slot + (long long)it_ * g_n) * 32 + rl;
    if (r > M - 1) r = M - 1;  // rows past the end repeat the last row and are never stored
    char* dst = lds + buf_ * kResTileBytes + wave * 1024;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (8 * i < 2 * NS && wave + 8 * i < 2 * NS && valid[i])
        __builtin_amdgcn_global_load_lds((gptr_t)(pb[i] + r * K), (lptr_t)(dst + i * 8192), 16, 0, 0);
  };
  const unsigned lds0 = (unsigned)(size_t)(lptr_t)lds;
  const unsigned la_row = lds0 + ll * 64 + ((h ^ ((ll >> 2) & 3)) * 16);
  // Stores of a finished block: a uniform row base per accumulator register plus one lane offset (column, and
  // the four rows that separate the wavefront's halves), so that the addresses cost no vector registers.
  const unsigned lane_off = (unsigned)(4 * h * N + col);
  auto store = [&](const floatx16& acc, int it_) {
    const long long row0 = ((long long)slot + (long long)it_ * g_n) * 32;
    float* yb = a.y + row0 * N;
    if (row0 + 32 <= M) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float v = acc[r] + bias;
        if (a.relu) v = v > 0.f ? v : 0.f;
        (yb + (size_t)(8 * (r >> 2) + (r & 3)) * N)[lane_off] = v;
      }
    } else {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float v = acc[r] + bias;
        if (a.relu) v = v > 0.f ? v : 0.f;
        if (row0 + 8 * (r >> 2) + 4 * h + (r & 3) < M) (yb + (size_t)(8 * (r >> 2) + (r & 3)) * N)[lane_off] = v;
      }
    }
  };
// One block: wait for its rows (requested two blocks ago, so they have long arrived; the wait also covers
// the previous block's stores, issued most of a block ago), then multiply it.  Requesting the block after
// next (into the buffer that every wavefront has finished reading) and storing the previous block are done
// at the start by wavefronts 0..3 and half-way through the contraction by wavefronts 4..7: the two
// wavefronts that share a SIMD then never leave the matrix pipe idle at the same time.
#define DCI_R_SIDE(IT, PREV)                                             \
  do {                                                                   \
    if ((IT) + 2 < n_my) issue((IT) + 2, ((IT) + 2) % kResBufs);         \
    if ((IT) > 0) store(PREV, (IT)-1);                                   \
  } while (0)
#define DCI_R_BLOCK(IT, ACC, PREV)                                       \
  do {                                                                   \
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                     \
    __builtin_amdgcn_s_barrier();                                        \
    const unsigned la0 = la_row + ((IT) % kResBufs) * kResTileBytes;     \
    const unsigned la1 = la0 ^ 32u;                                      \
    FragR f0, f1;                                                        \
    DCI_R_READ(f0, 0);                                                   \
    if (wave < 4) DCI_R_SIDE(IT, PREV);                                  \
    _Pragma("unroll") for (int r = 0; r < 16; ++r) ACC[r] = 0.f;         \
    DCI_R_SLAB(0, f0, f1, ACC) DCI_R_SLAB(1, f1, f0, ACC) DCI_R_SLAB(2, f0, f1, ACC) DCI_R_SLAB(3, f1, f0, ACC)     \
    DCI_R_SLAB(4, f0, f1, ACC) DCI_R_SLAB(5, f1, f0, ACC) DCI_R_SLAB(6, f0, f1, ACC) DCI_R_SLAB(7, f1, f0, ACC)     \
    if (wave >= 4) DCI_R_SIDE(IT, PREV);                                 \
    DCI_R_SLAB(8, f0, f1, ACC) DCI_R_SLAB(9, f1, f0, ACC) DCI_R_SLAB(10, f0, f1, ACC) DCI_R_SLAB(11, f1, f0, ACC)   \
    DCI_R_SLAB(12, f0, f1, ACC) DCI_R_SLAB(13, f1, f0, ACC) DCI_R_SLAB(14, f0, f1, ACC) DCI_R_SLAB(15, f1, f0, ACC) \
  } while (0)

  __syncthreads();  // the zero fill is complete before the first rows arrive
  issue(0, 0);
  if (n_my > 1) issue(1, 1);

  // This wavefront's weights.  Matrix step (T, j), T = 2 slab + t, takes chunk 2T of the padded sequence from
  // lanes 0..31 and chunk 2T + 1 from lanes 32..63, element j of each: lane (column ll, half h) keeps
  // W_op[4 (kc + h) + j][col], kc = 2T - op kpc.  Everything but the lane's byte offset is uniform, so a load
  // is a scalar row base plus one vector offset; every load is issued (from a row that exists) and the lanes
  // whose chunk is padding are zeroed afterwards.
  const unsigned off_pair = lane_off * 4u, off_first = (unsigned)col * 4u;
  float breg[8 * NS];
#pragma unroll
  for (int T = 0; T < 2 * NS; ++T) {
    const int op = 2 * T >= kpc ? 1 : 0;
    const int kc = 2 * T - op * kpc;                        // even
    const bool first_ok = op < n_ops && kc < kc_op;         // the pair's first chunk holds data
    const bool pair_ok = op < n_ops && kc + 1 < kc_op;      // and so does its second
    const char* wrow = reinterpret_cast<const char*>(first_ok ? (op ? a.w_neigh : W0) + (size_t)(4 * kc) * N : W0);
    const unsigned off = pair_ok ? off_pair : off_first;
#pragma unroll
    for (int j = 0; j < 4; ++j) breg[4 * T + j] = *reinterpret_cast<const float*>(wrow + (size_t)j * N * 4 + off);
  }
  // (a second pass, so that no load waits for the one before it)
#pragma unroll
  for (int T = 0; T < 2 * NS; ++T) {
    const int op = 2 * T >= kpc ? 1 : 0;
    const int kc = 2 * T - op * kpc;
    const bool first_ok = op < n_ops && kc < kc_op, pair_ok = op < n_ops && kc + 1 < kc_op;
    if (!pair_ok) {  // uniform, and false for all but the last pair or two of an operand
      const bool keep = first_ok && h == 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) breg[4 * T + j] = keep ? breg[4 * T + j] : 0.f;
    }
  }

  floatx16 acc_e, acc_o;
  for (int it = 0; it < n_my; it += 2) {
    DCI_R_BLOCK(it, acc_e, acc_o);
    if (it + 1 < n_my) DCI_R_BLOCK(it + 1, acc_o, acc_e);
  }
  if ((n_my - 1) & 1) store(acc_o, n_my - 1);
  else store(acc_e, n_my - 1);
#undef DCI_R_BLOCK
#undef DCI_R_SIDE
}

// ---- input layer in one kernel: aggregation inside the weights-in-registers dense layer ---------------
// k_sage_linear_res reads, per 32-row block, the self rows and the aggregated rows side by side from LDS.
// Here the aggregated half of a block is not loaded from a matrix that another kernel wrote: the workgroup
// computes it itself, one block ahead, while its matrix instructions run - the matrix pipe leaves the issue
// slots of a wavefront idle between dependent instructions, and the aggregation is loads plus a few additions.
// Every wavefront aggregates four rows of the next block (rows 4w .. 4w+3): half h of the wavefront sums one
// row, a lane of the half one 16-byte chunk of it, edge after edge in edge order (the order k_sage_mean uses,
// so the two routes agree to the bit).  The loads run as a fixed pipeline of 32 "slots" per block (2 row pairs
// x 16 edges): slot P is consumed eight slots after it was issued, so eight 16-byte loads per lane are in flight
// all the time; slots of edges a row does not have load a dummy line and add zero, which keeps the number of
// memory operations per block fixed (the wait before a block's barrier counts them).  Where a row's edges come
// from (cache slot or staged row, via blk_src and rowref) is worked out three blocks ahead and kept in LDS.
// Rows with more than 16 edges take the rest in a plain loop when the row is finished.
// Needs what k_sage_linear_res needs, two operands of at most 128 columns, and the mean or sum aggregator.
constexpr int kFuseSlots = 32, kFuseFan = 16, kFuseRing = 4;
__device__ float4 kFuseZeros[64] = {};  // what the slot of an edge that does not exist loads (one line per lane group, always zero)
struct FuseNote {               // per wavefront and block, in LDS
  unsigned long long base[64];  // lane 16 q + e: address of the source row of edge e of the wavefront's row q
  long long lo[4];              // first edge of row q
  int cnt[4];                   // edges of row q (0 for a row beyond the end)
  int pad[4];
};
struct FuseArgs {
  const long long* blk_indptr;
  const int* blk_src;
  const int* rowref;    // nullable: cache slot of a source, or -1
  const float* cache;   // rows of cached sources
  const float* x_src;   // rows of the other sources, by local id
  int mode;             // DCI_MODEL_SAGE_MEAN or DCI_MODEL_SAGE_SUM
};

template <int NS>
__global__ __launch_bounds__(kResThreads, 1) void k_sage_input_res(LinearArgs a, FuseArgs fa, int g_n) {
  static_assert(NS >= 4 && NS <= kResMaxSlabs, "slab count");
  // slots in flight per lane: eight where the registers allow it (the weights of the longest contraction take 128)
  constexpr int kFuseAhead = NS > 13 ? 4 : 8;
  __shared__ __attribute__((aligned(1024))) char lds[kResBufs * kResTileBytes];
  __shared__ FuseNote notes[kFuseRing][kResThreads / kWave];
  const long long M = a.counts[a.hop];
  const int id = (int)blockIdx.x;
  const int nt = id % a.n_tiles_n, slot = id / a.n_tiles_n;
  const long long n_rb = (M + 31) / 32;
  if (slot >= n_rb) return;
  const int n_my = (int)((n_rb - slot + g_n - 1) / g_n);
  const int tid = (int)threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int h = lane >> 5, ll = lane & 31;
  const int K = a.K, N = a.N;
  const int kc_op = K / 4;           // chunks of an operand that hold data (at most 32)
  const int kpc = (kc_op + 1) & ~1;  // chunks per operand in the padded sequence

  if (2 * kc_op != 4 * NS)
    for (int i = tid; i < kResBufs * kResTileBytes / 16; i += kResThreads)
      reinterpret_cast<float4*>(lds)[i] = make_float4(0.f, 0.f, 0.f, 0.f);

  const int col = nt * kResCols + wave * 32 + ll;
  const float bias = a.bias[col];

  // global->LDS loads of the self rows (operand 0 only: the other half of a block is computed here); the
  // addresses are formed when a block is requested rather than kept, registers being what this kernel is short of
  const int rl = 16 * (wave & 1) + (lane >> 2);
  const int c_a = (lane & 3) ^ ((lane >> 4) & 3);
  auto issue = [&](int it_, int buf_) {
    long long r = ((long long)slot + (long long)it_ * g_n) * 32 + rl;
    if (r > M - 1) r = M - 1;
    const float* prow = a.a_self + r * K + 4 * c_a;
    char* dst = lds + buf_ * kResTileBytes + wave * 1024;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (8 * i < 2 * NS && wave + 8 * i < 2 * NS && 4 * ((wave + 8 * i) >> 1) + c_a < kc_op)
        __builtin_amdgcn_global_load_lds((gptr_t)(prow + 16 * ((wave + 8 * i) >> 1)), (lptr_t)(dst + i * 8192), 16, 0, 0);
  };
  const unsigned lds0 = (unsigned)(size_t)(lptr_t)lds;
  const unsigned la_row = lds0 + ll * 64 + ((h ^ ((ll >> 2) & 3)) * 16);
  const unsigned lane_off = (unsigned)(4 * h * N + col);
  auto store = [&](const floatx16& acc, int it_) {
    const long long row0 = ((long long)slot + (long long)it_ * g_n) * 32;
    float* yb = a.y + row0 * N;
    if (row0 + 32 <= M) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float v = acc[r] + bias;
        if (a.relu) v = v > 0.f ? v : 0.f;
        (yb + (size_t)(8 * (r >> 2) + (r & 3)) * N)[lane_off] = v;
      }
    } else {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float v = acc[r] + bias;
        if (a.relu) v = v > 0.f ? v : 0.f;
        if (row0 + 8 * (r >> 2) + 4 * h + (r & 3) < M) (yb + (size_t)(8 * (r >> 2) + (r & 3)) * N)[lane_off] = v;
      }
    }
  };

  // ---- where the edges' rows are: worked out per block in four steps, each waiting for the one before ----
  struct Ix {
    int lo, hi;  // edge numbers stay below 2^31 (the batch bounds are checked against that)
    int s, rr;
    bool on;
  };
  auto index_bounds = [&](Ix& ix, int t) {
    const long long R = ((long long)slot + (long long)t * g_n) * 32 + 4 * wave + (lane >> 4);
    const bool ok = t < n_my && R < M;
    ix.lo = ok ? (int)fa.blk_indptr[R] : 0;
    ix.hi = ok ? (int)fa.blk_indptr[R + 1] : 0;
  };
  auto index_source = [&](Ix& ix) {
    ix.on = (lane & 15) < ix.hi - ix.lo;
    ix.s = ix.on ? fa.blk_src[(long long)ix.lo + (lane & 15)] : 0;
  };
  auto index_slot = [&](Ix& ix) { ix.rr = (ix.on && fa.rowref) ? fa.rowref[ix.s] : -1; };
  auto index_note = [&](const Ix& ix, int t) {
    FuseNote& nb = notes[t & (kFuseRing - 1)][wave];
    const float* p = ix.rr >= 0 ? fa.cache + (long long)ix.rr * K : fa.x_src + (long long)ix.s * K;
    nb.base[lane] = ix.on ? (unsigned long long)reinterpret_cast<uintptr_t>(p) : 0ull;
    if ((lane & 15) == 0) {
      nb.lo[lane >> 4] = ix.lo;
      nb.cnt[lane >> 4] = ix.hi - ix.lo;
    }
  };
  Ix ixs = {0, 0, 0, -1, false};  // the block being worked out while the matrix instructions run

  // ---- the slot pipeline ----
  float4v land[kFuseAhead];
  float4v agg = {0.f, 0.f, 0.f, 0.f};
  const float4v zero4 = {0.f, 0.f, 0.f, 0.f};
  const bool lane_on = ll < kc_op;
  const float* const zeros = reinterpret_cast<const float*>(kFuseZeros) + 4 * lane;
  auto slot_issue = [&](int t, int P) {  // P: 0 .. 31, a compile-time value at every call
    const FuseNote& nb = notes[t & (kFuseRing - 1)][wave];
    const int q = 2 * (P >> 4) + h, j = P & 15;
    const bool on = lane_on && j < nb.cnt[q];
    const float* p = on ? reinterpret_cast<const float*>((uintptr_t)nb.base[16 * q + j]) + 4 * ll : zeros;
    land[P & (kFuseAhead - 1)] = load_global_f4(p);
  };
  auto row_done = [&](int t, int rp) {  // the two rows of row pair rp of block t are complete: write them to the block's buffer
    const FuseNote& nb = notes[t & (kFuseRing - 1)][wave];
    const int q = 2 * rp + h;
    const int cnt = nb.cnt[q];
    if (cnt > kFuseFan && lane_on) {  // the edges beyond the pipelined sixteen
      const long long lo = nb.lo[q];
      for (int e = kFuseFan; e < cnt; ++e) {
        const int sidx = fa.blk_src[lo + e];
        const int rr = fa.rowref ? fa.rowref[sidx] : -1;
        const float* p = rr >= 0 ? fa.cache + (long long)rr * K : fa.x_src + (long long)sidx * K;
        agg += load_global_f4(p + 4 * ll);
      }
    }
    const float fc = (float)cnt;
    const float4v r = (fa.mode == DCI_MODEL_SAGE_SUM || cnt == 0) ? agg : agg / fc;
    if (lane_on) {
      const int row = 4 * wave + q;
      const int ck = kpc + ll;  // chunk of the second operand in the padded sequence
      char* dst = lds + (t % kResBufs) * kResTileBytes + (ck >> 2) * 2048 + row * 64 + (((ck & 3) ^ ((row >> 2) & 3)) * 16);
      *reinterpret_cast<float4v*>(dst) = r;
    }
    agg = zero4;
  };
  auto slot_take = [&](int t, int P) {
    agg += land[P & (kFuseAhead - 1)];
    if ((P & 15) == 15) row_done(t, P >> 4);
  };
// Slab S_ of the block that multiplies tile IT also handles slots kFuseSlots S_ / NS .. kFuseSlots (S_ + 1) / NS - 1 (two
// or three): it takes them from tile IT + 1 and issues the slots eight further on (of tile IT + 1, or of tile IT + 2 once
// past the end).  The slot work and the steps that find the sources of tile IT + 3 sit between the slab's matrix
// instructions, whose dependent chain leaves the wavefront's issue slots free.
#define DCI_F_SLOT(IT, S_, K_)                                                               \
  do {                                                                                       \
    constexpr int P_ = kFuseSlots * (S_) / NS + (K_);                                        \
    if (P_ < kFuseSlots * ((S_) + 1) / NS) {                                                 \
      slot_take((IT) + 1, P_);                                                               \
      if (P_ + kFuseAhead < kFuseSlots) slot_issue((IT) + 1, P_ + kFuseAhead);               \
      else slot_issue((IT) + 2, P_ + kFuseAhead - kFuseSlots);                               \
    }                                                                                        \
    __builtin_amdgcn_sched_barrier(0);                                                       \
  } while (0)
#define DCI_F_MFMA(FC_, E_, Q_, AC)                                                          \
  do {                                                                                       \
    AC = __builtin_amdgcn_mfma_f32_32x32x2f32(FC_ E_, breg[Q_], AC, 0, 0, 0);                \
    __builtin_amdgcn_sched_barrier(0);                                                       \
  } while (0)
#define DCI_F_SLAB(IT, S_, FC, FN, AC)                                                       \
  if ((S_) < NS) {                                                                           \
    DCI_R_WAIT(FC, 0);                                                                       \
    if ((S_) + 1 < NS) DCI_R_READ(FN, (((S_) + 1) % kResMaxSlabs) * 2048);                   \
    __builtin_amdgcn_sched_barrier(0);                                                       \
    DCI_F_MFMA(FC, .a0.x, 8 * (S_) + 0, AC);                                                 \
    DCI_F_SLOT(IT, S_, 0);                                                                   \
    DCI_F_MFMA(FC, .a0.y, 8 * (S_) + 1, AC);                                                 \
    DCI_F_MFMA(FC, .a0.z, 8 * (S_) + 2, AC);                                                 \
    DCI_F_SLOT(IT, S_, 1);                                                                   \
    DCI_F_MFMA(FC, .a0.w, 8 * (S_) + 3, AC);                                                 \
    DCI_F_MFMA(FC, .a1.x, 8 * (S_) + 4, AC);                                                 \
    DCI_F_SLOT(IT, S_, 2);                                                                   \
    DCI_F_MFMA(FC, .a1.y, 8 * (S_) + 5, AC);                                                 \
    if ((S_) == 0) index_bounds(ixs, (IT) + 3);                                              \
    if ((S_) == NS / 4) index_source(ixs);                                                   \
    if ((S_) == NS / 2) index_slot(ixs);                                                     \
    if ((S_) == (3 * NS) / 4) index_note(ixs, (IT) + 3);                                     \
    __builtin_amdgcn_sched_barrier(0);                                                       \
    DCI_F_MFMA(FC, .a1.z, 8 * (S_) + 6, AC);                                                 \
    DCI_F_MFMA(FC, .a1.w, 8 * (S_) + 7, AC);                                                 \
  }
// At the start of a block the newest memory operations of the wavefront are the previous block's (at most 16) stores
// and, before them, its eight slots in flight.  Every slot issues exactly one load, so the previous block issued at
// least 32 operations, all of them after this block's self rows were requested (two blocks ago): waiting for all but
// the newest 24 covers those rows whatever the stores were, and leaves the slots in flight.
#define DCI_F_BLOCK(IT)                                                  \
  do {                                                                   \
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(16 + kFuseAhead) : "memory"); \
    __builtin_amdgcn_s_barrier();                                        \
    const unsigned la0 = la_row + ((IT) % kResBufs) * kResTileBytes;     \
    const unsigned la1 = la0 ^ 32u;                                      \
    FragR f0, f1;                                                        \
    DCI_R_READ(f0, 0);                                                   \
    if (wave < 4 && (IT) + 2 < n_my) issue((IT) + 2, ((IT) + 2) % kResBufs); \
    floatx16 acc;                                                        \
    _Pragma("unroll") for (int r = 0; r < 16; ++r) acc[r] = 0.f;         \
    DCI_F_SLAB(IT, 0, f0, f1, acc) DCI_F_SLAB(IT, 1, f1, f0, acc) DCI_F_SLAB(IT, 2, f0, f1, acc) DCI_F_SLAB(IT, 3, f1, f0, acc)     \
    DCI_F_SLAB(IT, 4, f0, f1, acc) DCI_F_SLAB(IT, 5, f1, f0, acc) DCI_F_SLAB(IT, 6, f0, f1, acc) DCI_F_SLAB(IT, 7, f1, f0, acc)     \
    if (wave >= 4 && (IT) + 2 < n_my) issue((IT) + 2, ((IT) + 2) % kResBufs); \
    DCI_F_SLAB(IT, 8, f0, f1, acc) DCI_F_SLAB(IT, 9, f1, f0, acc) DCI_F_SLAB(IT, 10, f0, f1, acc) DCI_F_SLAB(IT, 11, f1, f0, acc)   \
    DCI_F_SLAB(IT, 12, f0, f1, acc) DCI_F_SLAB(IT, 13, f1, f0, acc) DCI_F_SLAB(IT, 14, f0, f1, acc) DCI_F_SLAB(IT, 15, f1, f0, acc) \
    store(acc, IT);                                                      \
  } while (0)

  __syncthreads();  // the zero fill is complete
  issue(0, 0);
  if (n_my > 1) issue(1, 1);

  // before the first block: where the rows of blocks 0, 1 and 2 come from; the whole of block 0's aggregated
  // half; the first eight slots of block 1 in flight
  {
    Ix p3[3];
#pragma unroll
    for (int t = 0; t < 3; ++t) index_bounds(p3[t], t);
#pragma unroll
    for (int t = 0; t < 3; ++t) index_source(p3[t]);
#pragma unroll
    for (int t = 0; t < 3; ++t) index_slot(p3[t]);
#pragma unroll
    for (int t = 0; t < 3; ++t) index_note(p3[t], t);
  }
#pragma unroll
  for (int P = 0; P < kFuseAhead; ++P) slot_issue(0, P);
#pragma unroll
  for (int P = 0; P < kFuseSlots; ++P) {
    slot_take(0, P);
    if (P + kFuseAhead < kFuseSlots) slot_issue(0, P + kFuseAhead);
    else slot_issue(1, P + kFuseAhead - kFuseSlots);
  }
  // this wavefront's weights (as in k_sage_linear_res), fetched after the first block's aggregation: together the two would not fit the registers
  const unsigned off_pair = lane_off * 4u, off_first = (unsigned)col * 4u;
  float breg[8 * NS];
#pragma unroll
  for (int T = 0; T < 2 * NS; ++T) {
    const int op = 2 * T >= kpc ? 1 : 0;
    const int kc = 2 * T - op * kpc;
    const bool first_ok = kc < kc_op, pair_ok = kc + 1 < kc_op;
    const char* wrow = reinterpret_cast<const char*>(first_ok ? (op ? a.w_neigh : a.w_self) + (size_t)(4 * kc) * N : a.w_self);
    const unsigned off = pair_ok ? off_pair : off_first;
#pragma unroll
    for (int j = 0; j < 4; ++j) breg[4 * T + j] = *reinterpret_cast<const float*>(wrow + (size_t)j * N * 4 + off);
  }

#pragma unroll
  for (int T = 0; T < 2 * NS; ++T) {
    const int op = 2 * T >= kpc ? 1 : 0;
    const int kc = 2 * T - op * kpc;
    const bool first_ok = kc < kc_op, pair_ok = kc + 1 < kc_op;
    if (!pair_ok) {
      const bool keep = first_ok && h == 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) breg[4 * T + j] = keep ? breg[4 * T + j] : 0.f;
    }
  }

  for (int it = 0; it < n_my; ++it) DCI_F_BLOCK(it);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the slots still in flight belong to no block
#undef DCI_F_BLOCK
#undef DCI_F_SLAB
#undef DCI_F_MFMA
#undef DCI_F_SLOT
}

// ---- input layer in one kernel, 64-row tiles: some wavefronts aggregate while the others multiply -------
// The other way to keep the aggregated rows out of HBM.  A workgroup (one per compute unit, eight wavefronts)
// walks 64-row tiles.  A tile's left operand - its self rows and its aggregated rows side by side, 64 rows x 2K,
// at most 64 KB - is built in LDS in the [slab][row][4 chunks] layout of k_sage_linear_dma by wavefronts 4 - 7:
// the self rows arrive by global->LDS loads; the aggregated rows they sum themselves (a half-wavefront per row, a
// lane per 16-byte chunk, edge after edge in edge order as k_sage_mean does).  These wavefronts keep no weights or
// accumulators, so their registers hold loads in flight: a row pair's sixteen 16-byte loads per lane and the first
// few of the next one's.
// Meanwhile wavefronts 0 - 3 multiply the tile built one step earlier (two such buffers) with the weights, one
// pass of 128 output columns after the other (32 per wavefront): every output element is one running sum over k in
// ascending order, as in k_sage_linear_res (so the one-kernel route and the two-kernel route that ends in that kernel
// agree to the bit), and every wavefront loads the weight values it needs straight into registers, several slabs ahead,
// so that the multiplying wavefronts never wait for each other and the whole workgroup meets at one barrier per tile.
// Needs two operands of K columns, 32 <= K <= 128, K a multiple of 16, an output width that is a multiple of 64,
// 16-byte aligned rows, weights, bias and output.
constexpr int kTileInThreads = 512, kTileInMaxSlabs = 16, kTileInFan = 16, kTileInAhead = 4;
constexpr int kTileInSlabBytes = TM * TK * 4;
constexpr int kTileInBufBytes = kTileInMaxSlabs * kTileInSlabBytes;  // 64 KB
constexpr int kTileInOutBytes = TM * 32 * 4;                         // a wavefront's 64 x 32 results on their way out
constexpr int kTileInLds = 2 * kTileInBufBytes + 4 * kTileInOutBytes;  // 160 KB

struct FragA {
  float4v a0, a1;  // rows 0 - 31 of the tile: four consecutive k of this lane's row, t = 0, 1
  float4v c0, c1;  // rows 32 - 63
};
#define DCI_T_READ(f, SLAB)                                                                            \
  asm volatile("ds_read_b128 %0, %4 offset:%6\n\tds_read_b128 %1, %5 offset:%6\n\t"                   \
               "ds_read_b128 %2, %4 offset:%7\n\tds_read_b128 %3, %5 offset:%7"                        \
               : "=&v"(f.a0), "=&v"(f.a1), "=&v"(f.c0), "=&v"(f.c1)                                    \
               : "v"(la0), "v"(la1), "n"((SLAB)*kTileInSlabBytes), "n"((SLAB)*kTileInSlabBytes + 2048) \
               : "memory")
#define DCI_T_WAIT(f)                                                              \
  do {                                                                             \
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");                             \
    asm volatile("" : "+v"(f.a0), "+v"(f.a1), "+v"(f.c0), "+v"(f.c1)::"memory");   \
  } while (0)

template <int SF>
__global__ __launch_bounds__(kTileInThreads, 1) void k_sage_input_tile(LinearArgs a, FuseArgs fa) {
  static_assert(SF >= 2 && 2 * SF <= kTileInMaxSlabs, "slabs per operand");
  __shared__ __attribute__((aligned(1024))) char lds[kTileInLds];
  const long long M = a.counts[a.hop];
  const long long n_tiles = (M + TM - 1) / TM;
  // Tiles blockIdx.x, + gridDim.x, ... in rounds.  The tiles of a last round that fills at most half of the workgroups
  // are taken by two workgroups each: both build the tile, each multiplies half of the passes over the output's
  // columns (the workgroups would otherwise idle for a whole tile while the others finish).
  const int n_pass = (a.N + 127) / 128;
  const int n_full = (int)(n_tiles / gridDim.x);
  const int rem = (int)(n_tiles - (long long)n_full * gridDim.x);
  const bool halves = n_pass >= 2 && rem > 0 && 2 * rem <= (int)gridDim.x;
  const bool has_last = halves ? (int)blockIdx.x < 2 * rem : (int)blockIdx.x < rem;
  const int n_my = n_full + (has_last ? 1 : 0);
  if (n_my == 0) return;
  const long long last_tile = (long long)n_full * gridDim.x + (halves ? (int)blockIdx.x >> 1 : (int)blockIdx.x);
  const int last_p0 = halves && (blockIdx.x & 1) ? n_pass / 2 : 0;
  const int last_p1 = halves && !(blockIdx.x & 1) ? n_pass / 2 : n_pass;
  const int tid = (int)threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int h = lane >> 5, ll = lane & 31;
  const int K = a.K, N = a.N;
  constexpr int Sf = SF;  // slabs per operand (K = 16 SF); a tile's slabs: 0 .. Sf-1 self rows, Sf .. 2 Sf-1 aggregated rows
  constexpr int n = 2 * Sf;

  // ---- the aggregated rows of a tile: row pairs RP0 .. RP1-1 of the sixteen rows 16 pw .. 16 pw + 15, two rows at a time
  // (one per half of the wavefront).  Every load is issued by every lane, from a line of zeros where there is nothing to
  // read: straight-line code, so that the loads of two row pairs are in flight together and only the oldest are waited for.
  const long long* const zeros_ll = reinterpret_cast<const long long*>(kFuseZeros);
  const int* const zeros_i = reinterpret_cast<const int*>(kFuseZeros);
  const float* const zeros_f = reinterpret_cast<const float*>(kFuseZeros) + 4 * lane;
  const bool lane_on = ll < K / 4;
  const float4v zero4 = {0.f, 0.f, 0.f, 0.f};
  auto aggregate = [&](char* const buf, const long long row0, const int pw, auto rp0_c, auto rp1_c) {
    constexpr int RP0 = decltype(rp0_c)::value, RP = decltype(rp1_c)::value - RP0;
    int lo[RP], cn[RP];
#pragma unroll
    for (int rp = 0; rp < RP; ++rp) {
      const long long R = row0 + 16 * pw + 2 * (RP0 + rp) + h;
      const long long* pb = R < M ? fa.blk_indptr + R : zeros_ll;
      const long long e0 = pb[0], e1 = pb[1];
      lo[rp] = (int)e0;  // edge numbers stay below 2^31 (the batch bounds are checked against that)
      cn[rp] = (int)(e1 - e0);
    }
    // lane e < 16 of a half: where the row of edge e of the half's row is
    int sidx[RP];
    bool on[RP];
#pragma unroll
    for (int rp = 0; rp < RP; ++rp) {
      on[rp] = ll < kTileInFan && ll < cn[rp];
      sidx[rp] = *(on[rp] ? fa.blk_src + ((long long)lo[rp] + ll) : zeros_i);
    }
    const float* bp[RP];
    if (fa.rowref) {
#pragma unroll
      for (int rp = 0; rp < RP; ++rp) {
        const int rr = *(on[rp] ? fa.rowref + sidx[rp] : zeros_i);
        bp[rp] = (on[rp] && rr >= 0) ? fa.cache + (long long)rr * K : fa.x_src + (long long)sidx[rp] * K;
      }
    } else {
#pragma unroll
      for (int rp = 0; rp < RP; ++rp) bp[rp] = fa.x_src + (long long)sidx[rp] * K;
    }
    float4v land[2][kTileInFan];
    auto request = [&](int rp, float4v* v, int j0, int j1) {  // slots j0 .. j1-1 of the row pair
#pragma unroll
      for (int j = 0; j < kTileInFan; ++j) {
        if (j < j0 || j >= j1) continue;
        const unsigned long long pj = __shfl((unsigned long long)reinterpret_cast<uintptr_t>(bp[rp]), (lane & 32) + j, kWave);
        const float* p = (lane_on && j < cn[rp]) ? reinterpret_cast<const float*>((uintptr_t)pj) + 4 * ll : zeros_f;
        v[j] = load_global_f4(p);
      }
    };
    auto finish = [&](int rp, const float4v* v) {
      float4v agg = zero4;
#pragma unroll
      for (int j = 0; j < kTileInFan; ++j) agg += v[j];  // slots beyond the row's edges hold zero
      const int cnt = cn[rp];
      if (cnt > kTileInFan && lane_on) {
        for (int e = kTileInFan; e < cnt; ++e) {
          const int s = fa.blk_src[(long long)lo[rp] + e];
          const int rr = fa.rowref ? fa.rowref[s] : -1;
          const float* p = rr >= 0 ? fa.cache + (long long)rr * K : fa.x_src + (long long)s * K;
          agg += load_global_f4(p + 4 * ll);
        }
      }
      const float fc = (float)cnt;
      const float4v r = (fa.mode == DCI_MODEL_SAGE_SUM || cnt == 0) ? agg : agg / fc;
      if (lane_on) {
        const int row = 16 * pw + 2 * (RP0 + rp) + h;
        char* dst = buf + (Sf + (ll >> 2)) * kTileInSlabBytes + row * 64 + (((ll & 3) ^ ((row >> 2) & 3)) * 16);
        *reinterpret_cast<float4v*>(dst) = r;
      }
    };
    // the next row pair's first kTileInAhead slots are requested before the current one is summed, the rest after:
    // 16 + kTileInAhead loads per lane in flight at most.  (Deeper queues only add to the latency that the other
    // wavefronts' weight loads see behind them.)
    request(0, land[0], 0, kTileInFan);
#pragma unroll
    for (int rp = 0; rp < RP; rp += 2) {
      request(rp + 1, land[1], 0, kTileInAhead);
      finish(rp, land[0]);
      request(rp + 1, land[1], kTileInAhead, kTileInFan);
      if (rp + 2 < RP) request(rp + 2, land[0], 0, kTileInAhead);
      finish(rp + 1, land[1]);
      if (rp + 2 < RP) request(rp + 2, land[0], kTileInAhead, kTileInFan);
    }
  };
  using rp_c0 = std::integral_constant<int, 0>;
  using rp_c4 = std::integral_constant<int, 4>;
  using rp_c8 = std::integral_constant<int, 8>;
  const long long row0_first = (n_full > 0 ? (long long)blockIdx.x : last_tile) * TM;

  if (wave >= 4) {
    // ================= building tiles =================
    const int pw = wave - 4;
    const int c_a = (lane & 3) ^ ((lane >> 4) & 3);
    for (int it = 0; it < n_my; ++it) {
      {
        char* const buf = lds + (it & 1) * kTileInBufBytes;
        const long long row0 = (it < n_full ? (long long)blockIdx.x + (long long)it * gridDim.x : last_tile) * TM;
        // self rows: this wave's sixteen rows of every slab (lane -> row, chunk of four k; chunk position xor-ed with row bits)
        {
          long long r_l = row0 + 16 * pw + (lane >> 2);
          if (r_l > M - 1) r_l = M - 1;
          const float* pa = a.a_self + r_l * K + 4 * c_a;
#pragma unroll
          for (int s = 0; s < Sf; ++s)
            __builtin_amdgcn_global_load_lds((gptr_t)(pa + TK * s), (lptr_t)(buf + s * kTileInSlabBytes + 1024 * pw), 16, 0, 0);
        }
        // the first tile's rows are shared with the multiplying wavefronts, which have nothing to multiply yet
        if (it == 0) aggregate(buf, row0, pw, rp_c0{}, rp_c4{});
        else aggregate(buf, row0, pw, rp_c0{}, rp_c8{});
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");  // the self rows have landed, the aggregated rows are written
      }
      __builtin_amdgcn_s_barrier();  // tile `it` is complete; the other wavefronts are done with the buffer of tile it - 1
    }
    return;
  }

  // ================= multiplying tiles =================
  // Wavefront w multiplies all 64 rows of the tile with 32 columns of the weights (columns 128 p + 32 w + 0..31 in pass
  // p over the output's columns): a weight value it loads serves two matrix instructions (rows 0 - 31 and 32 - 63).
  const unsigned lds0 = (unsigned)(size_t)(lptr_t)lds;
  const int cw = 32 * wave;
  // The weights go straight to registers: per slab and lane the eight values B[k][column] of its column, k = 4 h + 0..3
  // and 8 + 4 h + 0..3 (a load covers two k rows x 32 consecutive columns).  D register sets in rotation hold the slabs
  // to come; a slab is requested P = D - 2 steps before its turn into the set that was multiplied two steps ago (see
  // the note on fragment registers below; a global load is far slower than the two matrix instructions that can be
  // waiting).  D divides the slabs of a pass, so that a slab's set is the same in every pass and all register indices
  // are compile-time values.
  constexpr int D = n <= 8 ? n : n / 2, P = D - 2;
  static_assert(n % D == 0 && P >= 2, "rotation of the weight registers");
  const unsigned lane_off = (unsigned)(4 * h * N + ll);
  float bq[D][8];
  // q_s, q_c, q_it: the next slab to request, its pass's first column and its tile's number here (the wavefront
  // streams its tiles' passes one after the other; the weights depend on the pass only).  A wavefront whose columns lie beyond the output's width in the
  // last pass (N = 64 mod 128) loads columns 0 - 31 instead and stores nothing.
  int q_s = 0, q_it = 0, q_c = 128 * (n_full > 0 ? 0 : last_p0);
#define DCI_T_LOADB(SET)                                                                                       \
  do {                                                                                                         \
    const int qc_ = q_c + cw < N ? q_c + cw : 0;                                                               \
    const float* w_ = (q_s >= Sf ? a.w_neigh + (size_t)(q_s - Sf) * TK * N : a.w_self + (size_t)q_s * TK * N) + qc_; \
    gfptr_t wp_ = (gfptr_t)(w_ + lane_off); /* one pointer stepped from k row to k row: eight addresses would cost 16 registers */ \
    _Pragma("unroll") for (int j_ = 0; j_ < 8; ++j_) {                                                        \
      asm volatile("" : "+v"(wp_));                                                                            \
      bq[SET][j_] = *wp_;                                                                                      \
      wp_ += j_ == 3 ? 5 * (size_t)N : (size_t)N;                                                              \
    }                                                                                                          \
    if (++q_s == n) {                                                                                          \
      q_s = 0;                                                                                                 \
      q_c += 128;                                                                                              \
      if (q_c >= 128 * (q_it < n_full ? n_pass : last_p1)) { /* on to the next tile's first pass */            \
        ++q_it;                                                                                                \
        q_c = 128 * (q_it < n_full ? 0 : last_p0);                                                             \
      }                                                                                                        \
    }                                                                                                          \
  } while (0)
// Per output element one running sum over k in ascending order, as in k_sage_linear_res; the two row blocks alternate,
// so that a matrix instruction never waits for the one just before it.
#define DCI_T_MFMA(f, SET)                                                                 \
  do {                                                                                     \
    __builtin_amdgcn_sched_barrier(0);                                                     \
    acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a0.x, bq[SET][0], acc0, 0, 0, 0);        \
    acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(f.c0.x, bq[SET][0], acc1, 0, 0, 0);        \
    acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a0.y, bq[SET][1], acc0, 0, 0, 0);        \
    acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(f.c0.y, bq[SET][1], acc1, 0, 0, 0);        \
    acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a0.z, bq[SET][2], acc0, 0, 0, 0);        \
    acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(f.c0.z, bq[SET][2], acc1, 0, 0, 0);        \
    acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a0.w, bq[SET][3], acc0, 0, 0, 0);        \
    acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(f.c0.w, bq[SET][3], acc1, 0, 0, 0);        \
    acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a1.x, bq[SET][4], acc0, 0, 0, 0);        \
    acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(f.c1.x, bq[SET][4], acc1, 0, 0, 0);        \
    acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a1.y, bq[SET][5], acc0, 0, 0, 0);        \
    acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(f.c1.y, bq[SET][5], acc1, 0, 0, 0);        \
    acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a1.z, bq[SET][6], acc0, 0, 0, 0);        \
    acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(f.c1.z, bq[SET][6], acc1, 0, 0, 0);        \
    acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a1.w, bq[SET][7], acc0, 0, 0, 0);        \
    acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(f.c1.w, bq[SET][7], acc1, 0, 0, 0);        \
    __builtin_amdgcn_sched_barrier(0);                                                     \
  } while (0)
// Slab I of a pass, its row fragments in FC: request the weights of the slab P steps on (of the next pass or the next
// tile past the end of this one; LAST: the very last pass, where there is nothing further), read the next slab's row
// fragments if it belongs to this pass (the next pass reads its first ones itself: after a barrier they come from
// the other buffer), multiply.
#define DCI_T_STEP(FC, FN, FP, I, LAST)                                                \
  if ((I) < n) {                                                                       \
    DCI_T_WAIT(FC);                                                                    \
    if (!(LAST) || (I) + P < n) DCI_T_LOADB(((I) + P) % D);                            \
    if ((I) + 1 < n) DCI_T_READ(FN, ((I) + 1) % kTileInMaxSlabs);                      \
    DCI_T_MFMA(FC, (I) % D);                                                           \
    asm volatile("" : "+v"(FP.a0), "+v"(FP.a1), "+v"(FP.c0), "+v"(FP.c1));             \
  }
// Three sets of fragment registers in rotation: a step's reads land where the matrix instructions of two steps before
// read, never in registers that instructions still waiting for the matrix pipe may have to read (each matrix instruction
// depends on an earlier one of the step in between, so those of two steps before are complete).  The empty statement
// after a step's matrix instructions keeps the previous step's set alive, so that the three really are three sets of
// registers.  A pass starts in f0 (whatever used f0 last is complete by then: the sums have been stored); its first read
// stands inside the pass's code, after the branch that selects it, because nothing - not even a register copy that the
// compiler places at a branch - may touch the registers between a read and its wait: the compiler takes the read's
// results for present as soon as the statement that issues it is over.
#define DCI_T_PASS(LAST)                                                                                          \
  do {                                                                                                            \
    DCI_T_READ(f0, 0);                                                                                            \
    DCI_T_STEP(f0, f1, f2, 0, LAST) DCI_T_STEP(f1, f2, f0, 1, LAST) DCI_T_STEP(f2, f0, f1, 2, LAST)               \
    DCI_T_STEP(f0, f1, f2, 3, LAST) DCI_T_STEP(f1, f2, f0, 4, LAST) DCI_T_STEP(f2, f0, f1, 5, LAST)               \
    DCI_T_STEP(f0, f1, f2, 6, LAST) DCI_T_STEP(f1, f2, f0, 7, LAST) DCI_T_STEP(f2, f0, f1, 8, LAST)               \
    DCI_T_STEP(f0, f1, f2, 9, LAST) DCI_T_STEP(f1, f2, f0, 10, LAST) DCI_T_STEP(f2, f0, f1, 11, LAST)             \
    DCI_T_STEP(f0, f1, f2, 12, LAST) DCI_T_STEP(f1, f2, f0, 13, LAST) DCI_T_STEP(f2, f0, f1, 14, LAST)            \
    DCI_T_STEP(f0, f1, f2, 15, LAST)                                                                              \
  } while (0)

  // Nothing to multiply yet: this wavefront sums the second half of the rows of the first tile that wavefront 4 + wave
  // is building (its registers are free for the loads until the weights come in).
  aggregate(lds, row0_first, wave, rp_c4{}, rp_c8{});
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");  // those rows are written before the first barrier below
  FragA f0 = {}, f1 = {}, f2 = {};
#pragma unroll
  for (int i = 0; i < P; ++i) DCI_T_LOADB(i);  // slabs 0 .. P-1 of the first pass
  for (int it = 0; it < n_my; ++it) {
    const long long row0 = (it < n_full ? (long long)blockIdx.x + (long long)it * gridDim.x : last_tile) * TM;
    const int p0 = it < n_full ? 0 : last_p0, p1 = it < n_full ? n_pass : last_p1;
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // this wavefront's reads of the previous tile's buffer are complete
    __builtin_amdgcn_s_barrier();                        // tile `it` is in its buffer
    const unsigned la0 = lds0 + (it & 1) * kTileInBufBytes + ll * 64 + ((h ^ ((ll >> 2) & 3)) * 16);
    const unsigned la1 = la0 ^ 32u;
    for (int pass = p0; pass < p1; ++pass) {
      floatx16 acc0, acc1;  // rows 0 - 31 and 32 - 63
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        acc0[r] = 0.f;
        acc1[r] = 0.f;
      }
      // the pass's bias values, asked for now: at the end of the pass they would be a memory round trip on the critical path
      const int c4 = 4 * (lane & 7);
      const bool cols_ok = pass * 128 + cw < N;
      const int colb = cols_ok ? pass * 128 + cw + c4 : c4;
      const float4v b4 = *reinterpret_cast<const float4v*>(a.bias + colb);
      if (it == n_my - 1 && pass == p1 - 1) DCI_T_PASS(true);
      else DCI_T_PASS(false);
      // Out through the wavefront's own 8 KB of LDS, so that a lane stores 16 bytes of a row: eight stores per pass
      // instead of 32.  The wavefront's memory operations retire in order, so a wait for a weight load also waits for
      // every store before it; 32 stores between the loads would fill the counter and hold the next pass up for as
      // long as the stores take.
      if (cols_ok) {
        float* const ob = reinterpret_cast<float*>(lds + 2 * kTileInBufBytes + wave * kTileInOutBytes);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = 8 * (r >> 2) + 4 * h + (r & 3);
          ob[row * 32 + ll] = acc0[r];
          ob[(row + 32) * 32 + ll] = acc1[r];
        }
        typedef __attribute__((address_space(1))) float4v* gy4ptr_t;
        __attribute__((address_space(1))) float* yp = (__attribute__((address_space(1))) float*)(a.y + (row0 + (lane >> 3)) * N + colb);
        asm volatile("" : "+v"(yp));  // keeps the compiler from holding eight row addresses in registers from tile start on
        const size_t N8 = (size_t)N * 8;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int row = 8 * i + (lane >> 3);
          float4v v = *reinterpret_cast<const float4v*>(ob + row * 32 + c4) + b4;
          if (a.relu) {
            v.x = v.x > 0.f ? v.x : 0.f;
            v.y = v.y > 0.f ? v.y : 0.f;
            v.z = v.z > 0.f ? v.z : 0.f;
            v.w = v.w > 0.f ? v.w : 0.f;
          }
          if (row0 + row < M) *(gy4ptr_t)(yp) = v;
          yp += N8;
        }
      }
    }
  }
#undef DCI_T_PASS
#undef DCI_T_STEP
#undef DCI_T_MFMA
#undef DCI_T_LOADB
}
#undef DCI_T_READ
#undef DCI_T_WAIT

struct SageWs {
  float* m;
  float* y[2];
  float* part;         // partial sums of split dense layers
};

// How many workgroups share a tile of the 64x64 kernel: a layer with fewer tiles than compute units
// (small batches, narrow outputs) would walk the whole contraction in a handful of workgroups while
// the rest of the chip idles, so the contraction is cut into enough parts to put one workgroup on
// every compute unit.  More parts than that gain nothing: the kernel is bound by instruction issue,
// not by the latency of its slab chain.  tiles = launch size for the capacity, pairs = slab pairs.
constexpr int kSplitMaxTiles = 1024;  // no split beyond this many tiles (bounds the partial-sum planes)
static int split_for(int64_t tiles, int pairs, int num_cus) {
  if (tiles > kSplitMaxTiles) return 1;
  int64_t s = num_cus / tiles;
  if (s > 8) s = 8;
  if (s > pairs / 2) s = pairs / 2;  // at least two slab pairs per workgroup
  return s < 1 ? 1 : (int)s;
}

constexpr int kMaxCus = 304;  // upper bound used when sizing the workspace without a device at hand

static int64_t tile_rows8(int64_t cap) { return ((cap + TM - 1) / TM + 7) / 8 * 8; }

static void carve_sage_ws(Arena& ar, const int64_t* cap_rows, int32_t n_layers, const int32_t* dims, SageWs* ws) {
  size_t max_m = 1, max_y = 1, max_part = 1;
  for (int32_t l = 0; l < n_layers; ++l) {
    const int32_t h = n_layers - 1 - l;
    const size_t rows = (size_t)(cap_rows[h] > 0 ? cap_rows[h] : 1);
    if (rows * (size_t)dims[l] > max_m) max_m = rows * (size_t)dims[l];
    if (l != n_layers - 1 && rows * (size_t)dims[l + 1] > max_y) max_y = rows * (size_t)dims[l + 1];
    const int64_t tiles = tile_rows8((int64_t)rows) * ((dims[l + 1] + TN - 1) / TN);
    const int split = split_for(tiles, (dims[l] + TK - 1) / TK, kMaxCus);  // pairs of the two-operand layer; GCN has fewer and splits less
    if (split > 1) {
      const size_t need = (size_t)split * (size_t)tile_rows8((int64_t)rows) * TM * (size_t)dims[l + 1];
      if (need > max_part) max_part = need;
    }
  }
  ws->m = ar.take<float>(max_m);
  ws->y[0] = ar.take<float>(max_y);
  ws->y[1] = ar.take<float>(max_y);
  ws->part = ar.take<float>(max_part);
}

}  // namespace dci

using namespace dci;

extern "C" {

size_t dci_sage_workspace_bytes(const int64_t* cap_rows, int32_t n_layers, const int32_t* dims) {
  if (!cap_rows || !dims || n_layers < 1 || n_layers > DCI_MAX_HOPS) return 0;
  Arena ar(nullptr, 0);
  SageWs ws;
  carve_sage_ws(ar, cap_rows, n_layers, dims, &ws);
  return ar.off;
}

int32_t dci_sage_forward(dci_ctx* ctx, const dci_blocks* blocks, const float* x_in, int32_t n_layers,
                         const int32_t* dims, const float* const* w_self, const float* const* w_neigh,
                         const float* const* bias, float* logits) {
  return dci_gnn_forward(ctx, blocks, x_in, n_layers, dims, DCI_MODEL_SAGE_MEAN, w_self, w_neigh, bias, logits);
}

// Shared body of dci_gnn_forward and dci_gather_forward.  rowref != nullptr: the input layer's aggregation
// reads the row of source s from feat_cache[rowref[s]] when rowref[s] >= 0 and from x_in[s] otherwise.
// ws_off: bytes at the start of the workspace that the caller keeps for itself.
static int32_t forward_in(dci_ctx* ctx, const dci_blocks* blocks, const float* x_in, int32_t n_layers,
                          const int32_t* dims, int32_t model, const float* const* w_self,
                          const float* const* w_neigh, const float* const* bias, float* logits,
                          const int32_t* rowref, const float* feat_cache, size_t ws_off) {
  if (!ctx) return DCI_ERR_INVALID_ARG;
  if (model != DCI_MODEL_SAGE_MEAN && model != DCI_MODEL_SAGE_SUM && model != DCI_MODEL_GCN_AVG)
    return fail(ctx, DCI_ERR_INVALID_ARG, "gnn_forward: unknown model %d", model);
  const bool gcn = model == DCI_MODEL_GCN_AVG;
  if (!blocks || !blocks->counts || !x_in || !dims || (!gcn && !w_self) || !w_neigh || !bias || !logits)
    return fail(ctx, DCI_ERR_INVALID_ARG, "sage_forward: null argument");
  if (n_layers < 1 || n_layers > DCI_MAX_HOPS || n_layers != blocks->n_hops)
    return fail(ctx, DCI_ERR_INVALID_ARG, "sage_forward: n_layers must equal blocks.n_hops (1..%d)", DCI_MAX_HOPS);
  for (int32_t l = 0; l <= n_layers; ++l)
    if (dims[l] < 1) return fail(ctx, DCI_ERR_INVALID_ARG, "sage_forward: dims[%d] < 1", l);
  for (int32_t l = 0; l < n_layers; ++l)
    if ((!gcn && !w_self[l]) || !w_neigh[l] || !bias[l] || !blocks->blk_indptr[l] || !blocks->blk_src[l])
      return fail(ctx, DCI_ERR_INVALID_ARG, "sage_forward: null weight or block array at layer %d", l);
  Arena ar(ctx->ws, ctx->ws_bytes);
  if (ws_off) (void)ar.take<char>(ws_off);
  SageWs ws;
  carve_sage_ws(ar, blocks->cap_rows, n_layers, dims, &ws);
  if (!ar.ok())
    return fail(ctx, DCI_ERR_CAPACITY, "workspace holds %zu bytes, the forward pass needs %zu", ctx->ws_bytes, ar.off);
  const long long* counts = reinterpret_cast<const long long*>(blocks->counts);
  const float* x = x_in;
  auto aligned = [](const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; };
  for (int32_t l = 0; l < n_layers; ++l) {
    const int32_t h = n_layers - 1 - l;
    const int D = dims[l], Do = dims[l + 1];
    const int64_t cap = blocks->cap_rows[h] > 0 ? blocks->cap_rows[h] : 1;
    float* y = l == n_layers - 1 ? logits : ws.y[l & 1];
    // Input layer in one kernel (aggregation inside the weights-in-registers dense layer) where the layer qualifies
    const bool ref_l = l == 0 && rowref != nullptr;
    bool fuse_in = false;
    if (l == 0 && !gcn && ctx->input_layer != 1 && (ctx->linear_kernel == 0 || ctx->linear_kernel == 4)) {
      const int n_tiles_f = Do / kResCols;
      const bool shape_ok = Do % kResCols == 0 && D % 4 == 0 && D <= 128 && n_tiles_f > 0 && ctx->num_cus / n_tiles_f >= 1 &&
                            aligned(x, 16) && (!ref_l || aligned(feat_cache, 16));
      // By default only where it was measured ahead of the two kernels: up to 13 slabs (large's 2 x 100 columns: 107 us
      // against 60 + 64).  With all 16 slabs (huge's 2 x 128) the weights leave room for four slots in flight per
      // lane, the loads no longer keep up, and the kernel takes as long as the two it replaces (160 us).
      const int slabs_f = (2 * ((D / 4 + 1) & ~1) + 3) / 4;
      fuse_in = shape_ok && (ctx->input_layer == 2 || (ctx->linear_kernel == 0 && cap >= kResMinRows && slabs_f <= 13));
    }
    // The 64-row-tile form of the same: aggregate into LDS, then multiply (k_sage_input_tile)
    bool tile_in = false;
    if (l == 0 && !gcn && !fuse_in && (ctx->input_layer == 3 || ctx->input_layer == 0) && (ctx->linear_kernel == 0 || ctx->linear_kernel == 4)) {
      const bool shape_ok = Do % TN == 0 && D % TK == 0 && D >= 2 * TK && D <= 128 && aligned(x, 16) && (!ref_l || aligned(feat_cache, 16)) &&
                            aligned(w_self[l], 16) && aligned(w_neigh[l], 16) && aligned(y, 16) && aligned(bias[l], 16) && (cap + TM - 1) / TM < ((int64_t)1 << 31);
      tile_in = shape_ok && (ctx->input_layer == 3 || (ctx->linear_kernel == 0 && cap >= kResMinRows));
    }
    if (tile_in) {
      LinearArgs la;
      la.counts = counts;
      la.hop = h;
      la.a_self = x;
      la.a_neigh = x;  // not read: the second operand is aggregated inside the kernel
      la.w_self = w_self[l];
      la.w_neigh = w_neigh[l];
      la.single = 0;
      la.bias = bias[l];
      la.y = y;
      la.K = D;
      la.N = Do;
      la.relu = l != n_layers - 1;
      la.n_tiles_n = Do / TN;
      la.split = 1;
      la.n_tiles = 0;
      la.part_rows = 0;
      la.part = nullptr;
      FuseArgs fa;
      fa.blk_indptr = reinterpret_cast<const long long*>(blocks->blk_indptr[h]);
      fa.blk_src = blocks->blk_src[h];
      fa.rowref = ref_l ? rowref : nullptr;
      fa.cache = feat_cache;
      fa.x_src = x;
      fa.mode = model;
      {
        Timed timed(ctx, DCI_K_LINEAR_IN);
        const int64_t tiles_cap = (cap + TM - 1) / TM;
        const dim3 grid_t((unsigned)(tiles_cap < ctx->num_cus ? tiles_cap : ctx->num_cus));
        switch (D / TK) {
          case 2: hipLaunchKernelGGL(k_sage_input_tile<2>, grid_t, dim3(kTileInThreads), 0, ctx->stream, la, fa); break;
          case 3: hipLaunchKernelGGL(k_sage_input_tile<3>, grid_t, dim3(kTileInThreads), 0, ctx->stream, la, fa); break;
          case 4: hipLaunchKernelGGL(k_sage_input_tile<4>, grid_t, dim3(kTileInThreads), 0, ctx->stream, la, fa); break;
          case 5: hipLaunchKernelGGL(k_sage_input_tile<5>, grid_t, dim3(kTileInThreads), 0, ctx->stream, la, fa); break;
          case 6: hipLaunchKernelGGL(k_sage_input_tile<6>, grid_t, dim3(kTileInThreads), 0, ctx->stream, la, fa); break;
          case 7: hipLaunchKernelGGL(k_sage_input_tile<7>, grid_t, dim3(kTileInThreads), 0, ctx->stream, la, fa); break;
          default: hipLaunchKernelGGL(k_sage_input_tile<8>, grid_t, dim3(kTileInThreads), 0, ctx->stream, la, fa); break;
        }
      }
      DCI_LAUNCH_CHECK(ctx);
      x = y;
      continue;
    }
    if (fuse_in) {
      LinearArgs la;
      la.counts = counts;
      la.hop = h;
      la.a_self = x;
      la.a_neigh = x;  // not read: the second operand is aggregated inside the kernel
      la.w_self = w_self[l];
      la.w_neigh = w_neigh[l];
      la.single = 0;
      la.bias = bias[l];
      la.y = y;
      la.K = D;
      la.N = Do;
      la.relu = l != n_layers - 1;
      la.n_tiles_n = Do / kResCols;
      la.split = 1;
      la.n_tiles = 0;
      la.part_rows = 0;
      la.part = nullptr;
      FuseArgs fa;
      fa.blk_indptr = reinterpret_cast<const long long*>(blocks->blk_indptr[h]);
      fa.blk_src = blocks->blk_src[h];
      fa.rowref = ref_l ? rowref : nullptr;
      fa.cache = feat_cache;
      fa.x_src = x;
      fa.mode = model;
      const int g_f = ctx->num_cus / la.n_tiles_n;
      const int slabs = (2 * ((D / 4 + 1) & ~1) + 3) / 4;
      const dim3 grid_f((unsigned)(g_f * la.n_tiles_n));
      {
        Timed timed(ctx, DCI_K_LINEAR_IN);
        if (slabs <= 4)
          hipLaunchKernelGGL(k_sage_input_res<4>, grid_f, dim3(kResThreads), 0, ctx->stream, la, fa, g_f);
        else if (slabs <= 8)
          hipLaunchKernelGGL(k_sage_input_res<8>, grid_f, dim3(kResThreads), 0, ctx->stream, la, fa, g_f);
        else if (slabs <= 13)
          hipLaunchKernelGGL(k_sage_input_res<13>, grid_f, dim3(kResThreads), 0, ctx->stream, la, fa, g_f);
        else
          hipLaunchKernelGGL(k_sage_input_res<16>, grid_f, dim3(kResThreads), 0, ctx->stream, la, fa, g_f);
      }
      DCI_LAUNCH_CHECK(ctx);
      x = y;
      continue;
    }
    // mean aggregation
    int V = 1;
    const bool cache_al16 = !(l == 0 && rowref) || aligned(feat_cache, 16), cache_al8 = !(l == 0 && rowref) || aligned(feat_cache, 8);
    if (D % 4 == 0 && aligned(x, 16) && cache_al16) V = 4;
    else if (D % 2 == 0 && aligned(x, 8) && cache_al8) V = 2;
    const int chunks = D / V;
    int lpr_log2 = 0;
    while ((1 << lpr_log2) < chunks && lpr_log2 < 6) ++lpr_log2;
    const int rows_per_block = kMeanBlock >> lpr_log2;
    int64_t mb = (cap + rows_per_block - 1) / rows_per_block;
    if (mb > (int64_t)ctx->num_cus * 16) mb = (int64_t)ctx->num_cus * 16;
    const long long* bi = reinterpret_cast<const long long*>(blocks->blk_indptr[h]);
    {
    Timed timed(ctx, l == 0 ? DCI_K_MEAN_IN : DCI_K_MEAN);
    const bool ref = l == 0 && rowref != nullptr;
    const int* bsrc = (const int*)blocks->blk_src[h];
#define DCI_MEAN_LAUNCH(VV, RR, CC)                                                                                  \
  hipLaunchKernelGGL((k_sage_mean<VV, RR, CC>), dim3((int)mb), dim3(kMeanBlock), 0, ctx->stream, counts, h, bi, bsrc, \
                     x, D, lpr_log2, ws.m, model, (const int*)rowref, feat_cache)
#define DCI_MEAN_BY_CPL(VV, RR)                         \
  do {                                                  \
    switch (cpl) {                                      \
      case 1: DCI_MEAN_LAUNCH(VV, RR, 1); break;        \
      case 2: DCI_MEAN_LAUNCH(VV, RR, 2); break;        \
      case 3: DCI_MEAN_LAUNCH(VV, RR, 3); break;        \
      case 4: DCI_MEAN_LAUNCH(VV, RR, 4); break;        \
      case 5: DCI_MEAN_LAUNCH(VV, RR, 5); break;        \
      case 6: DCI_MEAN_LAUNCH(VV, RR, 6); break;        \
      case 7: DCI_MEAN_LAUNCH(VV, RR, 7); break;        \
      case 8: DCI_MEAN_LAUNCH(VV, RR, 8); break;        \
      default: DCI_MEAN_LAUNCH(VV, RR, 0); break;       \
    }                                                   \
  } while (0)
    const int cpl = (chunks + (1 << lpr_log2) - 1) >> lpr_log2;  // chunks per lane
    if (ref) {
      if (V == 4) DCI_MEAN_BY_CPL(4, true);
      else if (V == 2) DCI_MEAN_BY_CPL(2, true);
      else DCI_MEAN_BY_CPL(1, true);
    } else {
      if (V == 4) DCI_MEAN_BY_CPL(4, false);
      else if (V == 2) DCI_MEAN_BY_CPL(2, false);
      else DCI_MEAN_BY_CPL(1, false);
    }
#undef DCI_MEAN_BY_CPL
#undef DCI_MEAN_LAUNCH
    }
    DCI_LAUNCH_CHECK(ctx);
    // dense layer
    LinearArgs la;
    la.counts = counts;
    la.hop = h;
    la.a_self = x;
    la.a_neigh = ws.m;
    la.w_self = gcn ? w_neigh[l] : w_self[l];
    la.single = gcn ? 1 : 0;
    la.w_neigh = w_neigh[l];
    la.bias = bias[l];
    la.y = y;
    la.K = D;
    la.N = Do;
    la.relu = l != n_layers - 1;
    la.n_tiles_n = (Do + TN - 1) / TN;
    const int64_t m_tiles8 = tile_rows8(cap);  // row tiles, rounded up to whole XCD rounds
    const int64_t n_tiles = m_tiles8 * la.n_tiles_n;
    const int n_pairs = gcn ? ((D + TK - 1) / TK + 1) / 2 : (D + TK - 1) / TK;
    la.split = split_for(n_tiles, n_pairs, ctx->num_cus < kMaxCus ? ctx->num_cus : kMaxCus);
    if (ctx->linear_split > 0 && ctx->linear_split <= la.split) la.split = ctx->linear_split;
    la.n_tiles = (int)n_tiles;
    la.part_rows = m_tiles8 * TM;
    la.part = ws.part;
    const int64_t n_blocks = n_tiles * la.split;
    if (n_blocks >= ((int64_t)1 << 31)) return fail(ctx, DCI_ERR_UNSUPPORTED, "sage_forward: too many tiles");
    int va = 1;
    if (D % 4 == 0 && aligned(x, 16) && aligned(ws.m, 16)) va = 4;
    else if (D % 2 == 0 && aligned(x, 8) && aligned(ws.m, 8)) va = 2;
    const int vb = (Do % 4 == 0 && aligned(la.w_self, 16) && aligned(w_neigh[l], 16)) ? 4 : 1;
    dim3 grid((unsigned)n_blocks);  // tile kernel: tiles x parts of the contraction
    // wide kernel: 128-column tiles, 16-byte global->LDS loads (rows at least 8-byte aligned, weights
    // 16-byte aligned), one workgroup per compute unit; worth it once there are a few thousand rows
    const int n_tiles_w = Do / kWideCols;
    const int g_n = n_tiles_w > 0 ? (ctx->num_cus / 8 / n_tiles_w) * 8 : 0;
    const bool wide_ok = Do % kWideCols == 0 && D % 2 == 0 && g_n >= 8 && vb == 4 && aligned(x, 8) &&
                         aligned(ws.m, 8) && aligned(bias[l], 4);
    // weights in registers: short contractions (both operands together at most 256 long), 256-column tiles
    const int n_tiles_r = Do / kResCols;
    const int g_r = n_tiles_r > 0 ? ctx->num_cus / n_tiles_r : 0;
    const int res_chunks = (gcn ? 1 : 2) * ((D / 4 + 1) & ~1);  // chunks of four k, each operand padded to an even count
    const bool res_ok = Do % kResCols == 0 && D % 4 == 0 && res_chunks <= 4 * kResMaxSlabs && g_r >= 1 &&
                        aligned(x, 16) && aligned(ws.m, 16);
    const bool use_res = res_ok && (ctx->linear_kernel == 4 || (ctx->linear_kernel == 0 && cap >= kResMinRows));
    const bool use_wide = !use_res && wide_ok && (ctx->linear_kernel == 2 || (ctx->linear_kernel == 0 && cap >= kWideMinRows && D >= kWideMinWidth));
    // 64x64 tiles fed by global->LDS loads: unsplit layers whose widths and alignment allow it
    const bool dma_ok = Do % TN == 0 && D % 2 == 0 && vb == 4 && va >= 2 && la.split == 1;
    const bool use_dma = !use_res && !use_wide && dma_ok && (ctx->linear_kernel == 0 || ctx->linear_kernel == 3);
    {
      Timed timed(ctx, l == 0 ? DCI_K_LINEAR_IN : DCI_K_LINEAR);
      if (use_res) {
        la.n_tiles_n = n_tiles_r;
        const int slabs = (res_chunks + 3) / 4;
        const dim3 grid_r((unsigned)(g_r * n_tiles_r));
        if (slabs <= 4)
          hipLaunchKernelGGL(k_sage_linear_res<4>, grid_r, dim3(kResThreads), 0, ctx->stream, la, g_r);
        else if (slabs <= 8)
          hipLaunchKernelGGL(k_sage_linear_res<8>, grid_r, dim3(kResThreads), 0, ctx->stream, la, g_r);
        else if (slabs <= 13)
          hipLaunchKernelGGL(k_sage_linear_res<13>, grid_r, dim3(kResThreads), 0, ctx->stream, la, g_r);
        else
          hipLaunchKernelGGL(k_sage_linear_res<16>, grid_r, dim3(kResThreads), 0, ctx->stream, la, g_r);
      } else if (use_wide) {
        la.n_tiles_n = n_tiles_w;
        if (l == 0)
          hipLaunchKernelGGL(k_sage_linear_wide<true>, dim3((unsigned)(g_n * n_tiles_w)), dim3(kWideThreads), 0,
                             ctx->stream, la, g_n);
        else
          hipLaunchKernelGGL(k_sage_linear_wide<false>, dim3((unsigned)(g_n * n_tiles_w)), dim3(kWideThreads), 0,
                             ctx->stream, la, g_n);
      } else if (use_dma) {
        hipLaunchKernelGGL(k_sage_linear_dma, dim3((unsigned)n_tiles), dim3(kGemmThreads), 0, ctx->stream, la);
      } else if (va == 4 && vb == 4)
        hipLaunchKernelGGL((k_sage_linear<4, 4>), grid, dim3(kGemmThreads), 0, ctx->stream, la);
      else if (va == 4)
        hipLaunchKernelGGL((k_sage_linear<4, 1>), grid, dim3(kGemmThreads), 0, ctx->stream, la);
      else if (va == 2 && vb == 4)
        hipLaunchKernelGGL((k_sage_linear<2, 4>), grid, dim3(kGemmThreads), 0, ctx->stream, la);
      else if (va == 2)
        hipLaunchKernelGGL((k_sage_linear<2, 1>), grid, dim3(kGemmThreads), 0, ctx->stream, la);
      else if (vb == 4)
        hipLaunchKernelGGL((k_sage_linear<1, 4>), grid, dim3(kGemmThreads), 0, ctx->stream, la);
      else
        hipLaunchKernelGGL((k_sage_linear<1, 1>), grid, dim3(kGemmThreads), 0, ctx->stream, la);
      if (!use_res && !use_wide && !use_dma && la.split > 1) {
        int64_t rb = (cap * Do + 255) / 256;
        if (rb > (int64_t)ctx->num_cus * 8) rb = (int64_t)ctx->num_cus * 8;
        hipLaunchKernelGGL(k_split_reduce, dim3((unsigned)rb), dim3(256), 0, ctx->stream, la);
      }
    }
    DCI_LAUNCH_CHECK(ctx);
    x = y;
  }
  return DCI_OK;
}

int32_t dci_gnn_forward(dci_ctx* ctx, const dci_blocks* blocks, const float* x_in, int32_t n_layers,
                        const int32_t* dims, int32_t model, const float* const* w_self,
                        const float* const* w_neigh, const float* const* bias, float* logits) {
  return forward_in(ctx, blocks, x_in, n_layers, dims, model, w_self, w_neigh, bias, logits, nullptr, nullptr, 0);
}

static size_t gather_forward_prefix_bytes(const dci_ctx* ctx, int64_t cap_nodes, size_t* partials_off) {
  Arena ar(nullptr, 0);
  (void)ar.take<int32_t>((size_t)(cap_nodes > 0 ? cap_nodes : 1));
  *partials_off = ar.off;
  (void)ar.take<char>(ctx ? gather_partials_bytes(ctx) : (size_t)kMaxCus * 16 * 3 * sizeof(unsigned long long));
  return ar.off;
}

size_t dci_gather_forward_workspace_bytes(int64_t cap_nodes, const int64_t* cap_rows, int32_t n_layers,
                                          const int32_t* dims) {
  const size_t fwd = dci_sage_workspace_bytes(cap_rows, n_layers, dims);
  if (fwd == 0 || cap_nodes < 0) return 0;
  size_t unused;
  return gather_forward_prefix_bytes(nullptr, cap_nodes, &unused) + fwd;
}

int32_t dci_gather_forward(dci_ctx* ctx, const dci_graph* graph, const dci_cache* cache, const dci_blocks* blocks,
                           float* x, int32_t n_layers, const int32_t* dims, int32_t model,
                           const float* const* w_self, const float* const* w_neigh, const float* const* bias,
                           float* logits, uint64_t* stats) {
  if (!ctx) return DCI_ERR_INVALID_ARG;
  if (!graph || !graph->feat || graph->feat_dim < 1 || !blocks || !blocks->nodes || !blocks->counts || !x || !dims)
    return fail(ctx, DCI_ERR_INVALID_ARG, "gather_forward: null argument or missing feature matrix");
  if (n_layers < 1 || n_layers > DCI_MAX_HOPS || n_layers != blocks->n_hops)
    return fail(ctx, DCI_ERR_INVALID_ARG, "gather_forward: n_layers must equal blocks.n_hops (1..%d)", DCI_MAX_HOPS);
  if (dims[0] != graph->feat_dim)
    return fail(ctx, DCI_ERR_INVALID_ARG, "gather_forward: dims[0] = %d but the graph has %d features", dims[0], graph->feat_dim);
  if (cache && (!cache->feat_remap || (cache->feat_rows > 0 && !cache->feat_cache)))
    return fail(ctx, DCI_ERR_INVALID_ARG, "cache: null feature arrays");
  if ((reinterpret_cast<uintptr_t>(graph->feat) | reinterpret_cast<uintptr_t>(x) |
       (cache ? reinterpret_cast<uintptr_t>(cache->feat_cache) : 0)) & 3)
    return fail(ctx, DCI_ERR_INVALID_ARG, "feature arrays must be 4-byte aligned");
  size_t partials_off;
  const size_t prefix = gather_forward_prefix_bytes(ctx, blocks->cap_nodes, &partials_off);
  if (prefix > ctx->ws_bytes || !ctx->ws)
    return fail(ctx, DCI_ERR_CAPACITY, "workspace holds %zu bytes, gather_forward needs more than %zu", ctx->ws_bytes, prefix);
  int32_t* rowref = reinterpret_cast<int32_t*>(ctx->ws);
  // the rows the dense layer of the input layer reads as a matrix: F_{L-1}, a prefix of the input nodes
  const int64_t* n_dense = blocks->counts + (n_layers - 1);
  int32_t rc = gather_launch(ctx, graph, cache, blocks->nodes, blocks->cap_nodes, blocks->counts + n_layers, x, stats,
                             ctx->ws + partials_off, rowref, n_dense, blocks->cap_rows[n_layers - 1]);
  if (rc != DCI_OK) return rc;
  return forward_in(ctx, blocks, x, n_layers, dims, model, w_self, w_neigh, bias, logits, rowref,
                    cache ? cache->feat_cache : nullptr, prefix);
}

}  // extern "C"
