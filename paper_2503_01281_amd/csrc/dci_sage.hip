// GraphSAGE-mean forward over the blocks of one mini-batch (Table III family, mean aggregator).
//
// Per layer two kernels:
//   k_sage_mean   - m_i = mean of x[src] over row i of the block (bandwidth bound: one lane group
//                   per destination row, consecutive lanes on consecutive chunks of the row);
//   k_sage_linear - y = x W_self + m W_neigh + b (+ ReLU): one dense contraction over the
//                   concatenated K = 2*D axis on the matrix cores (v_mfma_f32_32x32x2f32, fp32 in,
//                   fp32 accumulate), 128x128 output tile per workgroup of four wavefronts,
//                   operands staged through LDS in k-major order so that fragment reads are
//                   conflict free.
// Row counts come from the block's device-side `counts`, so no host round trip is needed; the
// grids are sized for the capacities and surplus workgroups leave at once.
#include "dci_internal.h"

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

template <int V>
__global__ __launch_bounds__(kMeanBlock) void k_sage_mean(const long long* __restrict__ counts, int hop,
                                                          const long long* __restrict__ blk_indptr,
                                                          const int* __restrict__ blk_src,
                                                          const float* __restrict__ x, int D, int lpr_log2,
                                                          float* __restrict__ m) {
  typedef VecF<V> O;
  typedef typename O::type vec_t;
  const long long n_rows = counts[hop];
  const int chunks = D / V;
  const int lpr = 1 << lpr_log2;
  const int rows_per_block = kMeanBlock >> lpr_log2;
  const int sub = (int)threadIdx.x >> lpr_log2;
  const int cl = (int)threadIdx.x & (lpr - 1);
  for (long long base = (long long)blockIdx.x * rows_per_block; base < n_rows;
       base += (long long)gridDim.x * rows_per_block) {
    const long long i = base + sub;
    if (i >= n_rows) continue;
    const long long e0 = blk_indptr[i], e1 = blk_indptr[i + 1];
    const float cnt = (float)(e1 - e0);
    vec_t* dst = reinterpret_cast<vec_t*>(m + i * D);
    for (int c = cl; c < chunks; c += lpr) {
      vec_t acc = O::zero();
      long long e = e0;
      for (; e + 3 < e1; e += 4) {
        const int s0 = blk_src[e], s1 = blk_src[e + 1], s2 = blk_src[e + 2], s3 = blk_src[e + 3];
        const vec_t v0 = reinterpret_cast<const vec_t*>(x + (long long)s0 * D)[c];
        const vec_t v1 = reinterpret_cast<const vec_t*>(x + (long long)s1 * D)[c];
        const vec_t v2 = reinterpret_cast<const vec_t*>(x + (long long)s2 * D)[c];
        const vec_t v3 = reinterpret_cast<const vec_t*>(x + (long long)s3 * D)[c];
        O::add(acc, v0);
        O::add(acc, v1);
        O::add(acc, v2);
        O::add(acc, v3);
      }
      for (; e < e1; ++e) O::add(acc, reinterpret_cast<const vec_t*>(x + (long long)blk_src[e] * D)[c]);
      dst[c] = e1 > e0 ? O::div(acc, cnt) : O::zero();
    }
  }
}

// ---- dense layer on the matrix cores ---------------------------------------------------------
constexpr int BM = 128, BN = 128, BK = 16, LDS_PAD = 4;
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
};

__global__ __launch_bounds__(kGemmThreads) void k_sage_linear(LinearArgs a) {
  __shared__ float As[2][BK][BM + LDS_PAD];
  __shared__ float Bs[2][BK][BN + LDS_PAD];
  const long long M = a.counts[a.hop];
  const long long row0 = (long long)blockIdx.y * BM;
  const int col0 = (int)blockIdx.x * BN;
  if (row0 >= M) return;
  const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int K = a.K, N = a.N;
  const int kt_per_src = (K + BK - 1) / BK;
  const int n_kt = 2 * kt_per_src;

  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  float ra[8], rb[8];
  auto load_tile = [&](int kt) {
    const bool second = kt >= kt_per_src;
    const float* A = second ? a.a_neigh : a.a_self;
    const float* W = second ? a.w_neigh : a.w_self;
    const int k0 = (second ? kt - kt_per_src : kt) * BK;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int e = tid + kGemmThreads * q;
      const int ak = e & (BK - 1), ar = e >> 4;  // A: 16 consecutive k per row
      const long long row = row0 + ar;
      ra[q] = (row < M && k0 + ak < K) ? A[row * K + k0 + ak] : 0.f;
      const int bn = e & (BN - 1), bk = e >> 7;  // W: 128 consecutive n per k
      rb[q] = (k0 + bk < K && col0 + bn < N) ? W[(long long)(k0 + bk) * N + col0 + bn] : 0.f;
    }
  };
  auto store_tile = [&](int buf) {
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int e = tid + kGemmThreads * q;
      As[buf][e & (BK - 1)][e >> 4] = ra[q];
      Bs[buf][e >> 7][e & (BN - 1)] = rb[q];
    }
  };

  load_tile(0);
  store_tile(0);
  __syncthreads();
  for (int kt = 0; kt < n_kt; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < n_kt) load_tile(kt + 1);
#pragma unroll
    for (int kk = 0; kk < BK / 2; ++kk) {
      const int k = 2 * kk + (lane >> 5);
      float fa[2], fb[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        fa[t] = As[buf][k][wm * 64 + t * 32 + (lane & 31)];
        fb[t] = Bs[buf][k][wn * 64 + t * 32 + (lane & 31)];
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < n_kt) store_tile(buf ^ 1);
    __syncthreads();
  }

  // accumulator layout of the 32x32 tile: register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4,
  // column l%32.
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int col = col0 + wn * 64 + j * 32 + (lane & 31);
      if (col >= N) continue;
      const float b = a.bias[col];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const long long row = row0 + wm * 64 + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (row < M) {
          float v = acc[i][j][r] + b;
          if (a.relu) v = v > 0.f ? v : 0.f;
          a.y[row * N + col] = v;
        }
      }
    }
}

struct SageWs {
  float* m;
  float* y[2];
};

static void carve_sage_ws(Arena& ar, const int64_t* cap_rows, int32_t n_layers, const int32_t* dims, SageWs* ws) {
  size_t max_m = 1, max_y = 1;
  for (int32_t l = 0; l < n_layers; ++l) {
    const int32_t h = n_layers - 1 - l;
    const size_t rows = (size_t)(cap_rows[h] > 0 ? cap_rows[h] : 1);
    if (rows * (size_t)dims[l] > max_m) max_m = rows * (size_t)dims[l];
    if (l != n_layers - 1 && rows * (size_t)dims[l + 1] > max_y) max_y = rows * (size_t)dims[l + 1];
  }
  ws->m = ar.take<float>(max_m);
  ws->y[0] = ar.take<float>(max_y);
  ws->y[1] = ar.take<float>(max_y);
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
  if (!ctx) return DCI_ERR_INVALID_ARG;
  if (!blocks || !blocks->counts || !x_in || !dims || !w_self || !w_neigh || !bias || !logits)
    return fail(ctx, DCI_ERR_INVALID_ARG, "sage_forward: null argument");
  if (n_layers < 1 || n_layers > DCI_MAX_HOPS || n_layers != blocks->n_hops)
    return fail(ctx, DCI_ERR_INVALID_ARG, "sage_forward: n_layers must equal blocks.n_hops (1..%d)", DCI_MAX_HOPS);
  for (int32_t l = 0; l <= n_layers; ++l)
    if (dims[l] < 1) return fail(ctx, DCI_ERR_INVALID_ARG, "sage_forward: dims[%d] < 1", l);
  for (int32_t l = 0; l < n_layers; ++l)
    if (!w_self[l] || !w_neigh[l] || !bias[l] || !blocks->blk_indptr[l] || !blocks->blk_src[l])
      return fail(ctx, DCI_ERR_INVALID_ARG, "sage_forward: null weight or block array at layer %d", l);
  Arena ar(ctx->ws, ctx->ws_bytes);
  SageWs ws;
  carve_sage_ws(ar, blocks->cap_rows, n_layers, dims, &ws);
  if (!ar.ok())
    return fail(ctx, DCI_ERR_CAPACITY, "workspace holds %zu bytes, sage_forward needs %zu", ctx->ws_bytes, ar.off);
  const long long* counts = reinterpret_cast<const long long*>(blocks->counts);
  const float* x = x_in;
  auto aligned = [](const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; };
  for (int32_t l = 0; l < n_layers; ++l) {
    const int32_t h = n_layers - 1 - l;
    const int D = dims[l], Do = dims[l + 1];
    const int64_t cap = blocks->cap_rows[h] > 0 ? blocks->cap_rows[h] : 1;
    float* y = l == n_layers - 1 ? logits : ws.y[l & 1];
    // mean aggregation
    int V = 1;
    if (D % 4 == 0 && aligned(x, 16)) V = 4;
    else if (D % 2 == 0 && aligned(x, 8)) V = 2;
    const int chunks = D / V;
    int lpr_log2 = 0;
    while ((1 << lpr_log2) < chunks && lpr_log2 < 6) ++lpr_log2;
    const int rows_per_block = kMeanBlock >> lpr_log2;
    int64_t mb = (cap + rows_per_block - 1) / rows_per_block;
    if (mb > (int64_t)ctx->num_cus * 16) mb = (int64_t)ctx->num_cus * 16;
    const long long* bi = reinterpret_cast<const long long*>(blocks->blk_indptr[h]);
    {
    Timed timed(ctx, DCI_K_MEAN);
    if (V == 4)
      hipLaunchKernelGGL((k_sage_mean<4>), dim3((int)mb), dim3(kMeanBlock), 0, ctx->stream, counts, h, bi,
                         (const int*)blocks->blk_src[h], x, D, lpr_log2, ws.m);
    else if (V == 2)
      hipLaunchKernelGGL((k_sage_mean<2>), dim3((int)mb), dim3(kMeanBlock), 0, ctx->stream, counts, h, bi,
                         (const int*)blocks->blk_src[h], x, D, lpr_log2, ws.m);
    else
      hipLaunchKernelGGL((k_sage_mean<1>), dim3((int)mb), dim3(kMeanBlock), 0, ctx->stream, counts, h, bi,
                         (const int*)blocks->blk_src[h], x, D, lpr_log2, ws.m);
    }
    DCI_LAUNCH_CHECK(ctx);
    // dense layer
    LinearArgs la;
    la.counts = counts;
    la.hop = h;
    la.a_self = x;
    la.a_neigh = ws.m;
    la.w_self = w_self[l];
    la.w_neigh = w_neigh[l];
    la.bias = bias[l];
    la.y = y;
    la.K = D;
    la.N = Do;
    la.relu = l != n_layers - 1;
    dim3 grid((unsigned)((Do + BN - 1) / BN), (unsigned)((cap + BM - 1) / BM));
    if (grid.y > 65535u) return fail(ctx, DCI_ERR_UNSUPPORTED, "sage_forward: too many row tiles");
    {
      Timed timed(ctx, DCI_K_LINEAR);
      hipLaunchKernelGGL(k_sage_linear, grid, dim3(kGemmThreads), 0, ctx->stream, la);
    }
    DCI_LAUNCH_CHECK(ctx);
    x = y;
  }
  return DCI_OK;
}

}  // extern "C"
