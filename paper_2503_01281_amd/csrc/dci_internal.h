// Internal declarations shared by the HIP translation units of libdci (gfx950 only).
#ifndef DCI_INTERNAL_H_
#define DCI_INTERNAL_H_

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <cstring>

#include "dci.h"

struct dci_ctx {
  int device = 0;
  hipStream_t stream = nullptr;
  char* ws = nullptr;
  size_t ws_bytes = 0;
  char* static_scratch = nullptr;  // this GPU's copy of the library's static scratch array (DCI_STATIC_SCRATCH_BYTES)
  int num_cus = 256;
  hipEvent_t ev[3] = {nullptr, nullptr, nullptr};
  char err[512] = {0};
  // optional per-kernel-class timing
  uint32_t timing_mask = 0;
  hipEvent_t* t_events = nullptr;  // 2 * DCI_TIMING_MAX_LAUNCHES, created on first enable
  int8_t* t_class = nullptr;
  int t_used = 0;
  unsigned* host_flag = nullptr;  // pinned host word (64 bytes): a kernel raises it when a batch had to be voided
  unsigned relabel_spin_limit = 1u << 24;  // DCI_OPT_RELABEL_SPIN_LIMIT
  unsigned test_first_ticket = 0;          // DCI_OPT_TEST_RELABEL_FIRST_TICKET
  // what the last call that returned DCI_ERR_CAPACITY needed (dci_last_required)
  int64_t req_nodes[DCI_MAX_HOPS + 1] = {0};
  int64_t req_edges[DCI_MAX_HOPS] = {0};
  size_t req_workspace = 0;
  int relabel_tile_iters = 0;  // DCI_OPT_RELABEL_TILE_ITERS: 0 = by frontier size, else 2, 4 or 8 rows per lane group
  int input_layer = 0;    // DCI_OPT_INPUT_LAYER: 0 by shape, 1 aggregation and dense layer as two kernels, 2 / 3 one kernel where the shape allows (weights in registers / 64-row tiles)
  int fused_input = 0;    // DCI_OPT_FUSED_INPUT: dci_infer_batches lets the first layer read cached rows in place
  int linear_split = 0;   // DCI_OPT_LINEAR_SPLIT: 0 = by shape, n = at most n workgroups per tile
  int linear_kernel = 0;  // DCI_OPT_LINEAR_KERNEL: 0 by shape, 1 tile kernel, 2 wide kernel where the shape allows
};

namespace dci {

constexpr int kWave = 64;
constexpr size_t kAlign = 256;

inline int32_t fail(dci_ctx* ctx, int32_t code, const char* fmt, ...) {
  if (ctx) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
    va_end(ap);
  }
  return code;
}

#define DCI_HIP(ctx, call)                                                                          \
  do {                                                                                              \
    hipError_t e_ = (call);                                                                         \
    if (e_ != hipSuccess)                                                                           \
      return dci::fail((ctx), DCI_ERR_HIP, "%s failed: %s (%s:%d)", #call, hipGetErrorString(e_),   \
                       __FILE__, __LINE__);                                                         \
  } while (0)

#define DCI_LAUNCH_CHECK(ctx)                                                                       \
  do {                                                                                              \
    hipError_t e_ = hipGetLastError();                                                              \
    if (e_ != hipSuccess)                                                                           \
      return dci::fail((ctx), DCI_ERR_HIP, "kernel launch failed: %s (%s:%d)", hipGetErrorString(e_), \
                       __FILE__, __LINE__);                                                         \
  } while (0)

// Brackets the launches issued during its lifetime with a pair of events when the class is timed.
struct Timed {
  dci_ctx* ctx;
  int idx = -1;
  Timed(dci_ctx* c, int cls) : ctx(c) {
    if ((c->timing_mask >> cls) & 1u) {
      if (c->t_used < DCI_TIMING_MAX_LAUNCHES) {
        idx = c->t_used++;
        c->t_class[idx] = (int8_t)cls;
        (void)hipEventRecord(c->t_events[2 * idx], c->stream);
      }
    }
  }
  ~Timed() {
    if (idx >= 0) (void)hipEventRecord(ctx->t_events[2 * idx + 1], ctx->stream);
  }
};

inline size_t align_up(size_t x, size_t a = kAlign) { return (x + a - 1) / a * a; }

// Bump allocator over the context's workspace.  Every call carves its temporaries from the
// start: calls on one context are ordered on one stream, so they never hold it at the same time.
struct Arena {
  char* base;
  size_t cap;
  size_t off = 0;
  Arena(char* b, size_t c) : base(b), cap(c) {}
  template <class T>
  T* take(size_t n) {
    size_t bytes = align_up(n * sizeof(T));
    T* p = reinterpret_cast<T*>(base + off);
    off += bytes;
    return p;
  }
  bool ok() const { return off <= cap && (base != nullptr || off == 0); }
};

inline uint64_t next_pow2(uint64_t x) {
  uint64_t p = 1;
  while (p < x) p <<= 1;
  return p;
}

// -- device helpers -----------------------------------------------------------------------

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (kWave - 1)); }

__device__ __forceinline__ int wave_incl_scan(int x) {
  const int lane = lane_id();
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    int y = __shfl_up(x, d, kWave);
    if (lane >= d) x += y;
  }
  return x;
}

__device__ __forceinline__ long long wave_incl_scan64(long long x) {
  const int lane = lane_id();
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    long long y = __shfl_up(x, d, kWave);
    if (lane >= d) x += y;
  }
  return x;
}

__device__ __forceinline__ unsigned long long wave_sum_u64(unsigned long long x) {
#pragma unroll
  for (int d = kWave / 2; d >= 1; d >>= 1) x += __shfl_down(x, d, kWave);
  return x;  // valid in lane 0
}

// Fills `bytes` (a multiple of 16) at a 16-byte aligned address with the 32-bit pattern.
__global__ void k_fill_u32x4(uint4* __restrict__ p, size_t n16, uint32_t pattern);

int32_t fill_bytes(dci_ctx* ctx, void* p, size_t bytes, uint32_t pattern);
// After a wait on the context's stream: reports (and clears) a failure that a kernel flagged.
int32_t check_device_flag(dci_ctx* ctx);
// partials_buf: gather_partials_bytes(ctx) bytes of device scratch, needed when stats != NULL
// rowref / n_dense_dev: nullptr for the plain gather; otherwise the selective form (see k_gather_select),
// n_dense_max bounding *n_dense_dev
int32_t gather_launch(dci_ctx* ctx, const dci_graph* g, const dci_cache* cache, const int64_t* ids,
                      int64_t n_max, const int64_t* n_dev, float* out, uint64_t* stats, void* partials_buf,
                      int32_t* rowref, const int64_t* n_dense_dev, int64_t n_dense_max);
size_t gather_partials_bytes(const dci_ctx* ctx);

}  // namespace dci

#endif  // DCI_INTERNAL_H_
