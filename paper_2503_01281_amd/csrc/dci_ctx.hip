// Context management and small shared kernels of libdci.
#include "dci_internal.h"

#include <mutex>
#include <new>

// Temporaries of the entry points that may not allocate (dci_sample_khop_static): one array per GPU,
// held by that GPU from the moment the library's code is loaded on it until the process ends.
// In host code `scratch` only names the symbol; the address of a GPU's copy comes from
// hipGetSymbolAddress (scratch_for_device below) and is what every launch and fill is given.
static __device__ __align__(256) unsigned char scratch[DCI_STATIC_SCRATCH_BYTES];

namespace dci {

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices] = {nullptr};

// Address of `device`'s copy of the static scratch array; `device` must be the current device.
static hipError_t scratch_for_device(int device, void** out) {
  *out = nullptr;
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    void* p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p || (reinterpret_cast<uintptr_t>(p) % kAlign)) return hipErrorInvalidSymbol;
    g_scratch_ptr[device] = p;
  }
  *out = g_scratch_ptr[device];
  return hipSuccess;
}

__global__ void k_fill_u32x4(uint4* __restrict__ p, size_t n16, uint32_t pattern) {
  const uint4 v = make_uint4(pattern, pattern, pattern, pattern);
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x)
    p[i] = v;
}

// A fill kernel rather than hipMemsetAsync, so that callers may capture the calls in a graph.
int32_t fill_bytes(dci_ctx* ctx, void* p, size_t bytes, uint32_t pattern) {
  if (bytes == 0) return DCI_OK;
  if ((reinterpret_cast<uintptr_t>(p) & 15) || (bytes & 15))
    return fail(ctx, DCI_ERR_INVALID_ARG, "fill_bytes: unaligned region");
  const size_t n16 = bytes / 16;
  const int block = 256;
  size_t want = (n16 + block - 1) / block;
  const int grid = (int)(want < (size_t)ctx->num_cus * 8 ? want : (size_t)ctx->num_cus * 8);
  hipLaunchKernelGGL(k_fill_u32x4, dim3(grid), dim3(block), 0, ctx->stream, reinterpret_cast<uint4*>(p), n16,
                     pattern);
  DCI_LAUNCH_CHECK(ctx);
  return DCI_OK;
}

int32_t check_device_flag(dci_ctx* ctx) {
  if (ctx->host_flag && *ctx->host_flag != 0u) {
    *ctx->host_flag = 0u;
    return fail(ctx, DCI_ERR_HIP,
                "relabel scan timed out: a tile of the frontier scan waited longer than the spin limit for its "
                "predecessors; the batch was voided (sizes zeroed) and its outputs must not be used");
  }
  return DCI_OK;
}

}  // namespace dci

extern "C" {

int32_t dci_create(dci_ctx** out, int32_t device, void* hip_stream, void* workspace, size_t workspace_bytes) {
  if (!out) return DCI_ERR_INVALID_ARG;
  *out = nullptr;
  dci_ctx* ctx = new (std::nothrow) dci_ctx();
  if (!ctx) return DCI_ERR_HIP;
  ctx->device = device;
  ctx->stream = reinterpret_cast<hipStream_t>(hip_stream);
  hipError_t e = hipSetDevice(device);
  hipDeviceProp_t prop;
  if (e == hipSuccess) e = hipGetDeviceProperties(&prop, device);
  if (e == hipSuccess) {
    ctx->num_cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    for (int i = 0; i < 3 && e == hipSuccess; ++i) e = hipEventCreate(&ctx->ev[i]);
  }
  if (e == hipSuccess) {
    void* p = nullptr;
    e = dci::scratch_for_device(device, &p);
    ctx->static_scratch = static_cast<char*>(p);
  }
  if (e == hipSuccess) {
    void* p = nullptr;
    e = hipHostMalloc(&p, 64, hipHostMallocDefault);
    if (e == hipSuccess) {
      ctx->host_flag = static_cast<unsigned*>(p);
      *ctx->host_flag = 0u;
    }
  }
  if (e != hipSuccess) {
    for (int i = 0; i < 3; ++i)
      if (ctx->ev[i]) (void)hipEventDestroy(ctx->ev[i]);
    if (ctx->host_flag) (void)hipHostFree(ctx->host_flag);
    delete ctx;
    return DCI_ERR_HIP;
  }
  int32_t rc = dci_set_workspace(ctx, workspace, workspace_bytes);
  if (rc != DCI_OK) {
    dci_destroy(ctx);
    return rc;
  }
  *out = ctx;
  return DCI_OK;
}

int32_t dci_set_workspace(dci_ctx* ctx, void* workspace, size_t workspace_bytes) {
  if (!ctx) return DCI_ERR_INVALID_ARG;
  if ((workspace == nullptr) != (workspace_bytes == 0))
    return dci::fail(ctx, DCI_ERR_INVALID_ARG, "workspace pointer and size must both be set or both be empty");
  if (reinterpret_cast<uintptr_t>(workspace) % dci::kAlign)
    return dci::fail(ctx, DCI_ERR_INVALID_ARG, "workspace must be %zu-byte aligned", dci::kAlign);
  ctx->ws = static_cast<char*>(workspace);
  ctx->ws_bytes = workspace_bytes;
  return DCI_OK;
}

void dci_destroy(dci_ctx* ctx) {
  if (!ctx) return;
  if (ctx->host_flag) (void)hipHostFree(ctx->host_flag);
  for (int i = 0; i < 3; ++i)
    if (ctx->ev[i]) (void)hipEventDestroy(ctx->ev[i]);
  if (ctx->t_events) {
    for (int i = 0; i < 2 * DCI_TIMING_MAX_LAUNCHES; ++i)
      if (ctx->t_events[i]) (void)hipEventDestroy(ctx->t_events[i]);
    delete[] ctx->t_events;
  }
  delete[] ctx->t_class;
  delete ctx;
}

int32_t dci_timing_enable(dci_ctx* ctx, uint32_t class_mask) {
  if (!ctx) return DCI_ERR_INVALID_ARG;
  if (class_mask && !ctx->t_events) {
    ctx->t_events = new (std::nothrow) hipEvent_t[2 * DCI_TIMING_MAX_LAUNCHES]();
    ctx->t_class = new (std::nothrow) int8_t[DCI_TIMING_MAX_LAUNCHES]();
    if (!ctx->t_events || !ctx->t_class) return dci::fail(ctx, DCI_ERR_HIP, "out of host memory for timing events");
    for (int i = 0; i < 2 * DCI_TIMING_MAX_LAUNCHES; ++i) DCI_HIP(ctx, hipEventCreate(&ctx->t_events[i]));
  }
  ctx->timing_mask = class_mask;
  return DCI_OK;
}

int32_t dci_timing_read(dci_ctx* ctx, double* total_ms, int64_t* launches) {
  if (!ctx || !total_ms || !launches) return DCI_ERR_INVALID_ARG;
  for (int k = 0; k < DCI_K_COUNT; ++k) {
    total_ms[k] = 0.0;
    launches[k] = 0;
  }
  DCI_HIP(ctx, hipStreamSynchronize(ctx->stream));
  const int32_t flagged = dci::check_device_flag(ctx);
  for (int i = 0; i < ctx->t_used; ++i) {
    float ms = 0.f;
    DCI_HIP(ctx, hipEventElapsedTime(&ms, ctx->t_events[2 * i], ctx->t_events[2 * i + 1]));
    total_ms[ctx->t_class[i]] += ms;
    launches[ctx->t_class[i]] += 1;
  }
  ctx->t_used = 0;
  return flagged;
}

int32_t dci_sync(dci_ctx* ctx) {
  if (!ctx) return DCI_ERR_INVALID_ARG;
  DCI_HIP(ctx, hipStreamSynchronize(ctx->stream));
  return dci::check_device_flag(ctx);
}

const char* dci_last_error(const dci_ctx* ctx) { return ctx ? ctx->err : "null context"; }

int32_t dci_last_required(const dci_ctx* ctx, int64_t* cap_nodes, int64_t* cap_edges, size_t* workspace_bytes) {
  if (!ctx) return DCI_ERR_INVALID_ARG;
  if (cap_nodes) std::memcpy(cap_nodes, ctx->req_nodes, sizeof(ctx->req_nodes));
  if (cap_edges) std::memcpy(cap_edges, ctx->req_edges, sizeof(ctx->req_edges));
  if (workspace_bytes) *workspace_bytes = ctx->req_workspace;
  return DCI_OK;
}

int32_t dci_set_option(dci_ctx* ctx, int32_t option, int64_t value) {
  if (!ctx) return DCI_ERR_INVALID_ARG;
  if (option == DCI_OPT_LINEAR_KERNEL) {
    if (value < 0 || value > 4) return dci::fail(ctx, DCI_ERR_INVALID_ARG, "DCI_OPT_LINEAR_KERNEL takes 0 .. 4, not %lld", (long long)value);
    ctx->linear_kernel = (int)value;
    return DCI_OK;
  }
  if (option == DCI_OPT_LINEAR_SPLIT) {
    if (value < 0 || value > 8) return dci::fail(ctx, DCI_ERR_INVALID_ARG, "DCI_OPT_LINEAR_SPLIT takes 0..8, not %lld", (long long)value);
    ctx->linear_split = (int)value;
    return DCI_OK;
  }
  if (option == DCI_OPT_RELABEL_TILE_ITERS) {
    if (value != 0 && value != 2 && value != 4 && value != 8)
      return dci::fail(ctx, DCI_ERR_INVALID_ARG, "DCI_OPT_RELABEL_TILE_ITERS takes 0, 2, 4 or 8, not %lld", (long long)value);
    ctx->relabel_tile_iters = (int)value;
    return DCI_OK;
  }
  if (option == DCI_OPT_INPUT_LAYER) {
    if (value < 0 || value > 3) return dci::fail(ctx, DCI_ERR_INVALID_ARG, "DCI_OPT_INPUT_LAYER takes 0 .. 3, not %lld", (long long)value);
    ctx->input_layer = (int)value;
    return DCI_OK;
  }
  if (option == DCI_OPT_FUSED_INPUT) {
    if (value != 0 && value != 1) return dci::fail(ctx, DCI_ERR_INVALID_ARG, "DCI_OPT_FUSED_INPUT takes 0 or 1, not %lld", (long long)value);
    ctx->fused_input = (int)value;
    return DCI_OK;
  }
  if (option == DCI_OPT_RELABEL_SPIN_LIMIT) {
    if (value < 1 || value > (int64_t)0xFFFFFFFFll)
      return dci::fail(ctx, DCI_ERR_INVALID_ARG, "DCI_OPT_RELABEL_SPIN_LIMIT takes 1 .. 2^32-1, not %lld", (long long)value);
    if (ctx->test_first_ticket != 0 && value > 65536)
      return dci::fail(ctx, DCI_ERR_INVALID_ARG, "the spin limit must stay at or below 65536 while the first-ticket test hook is on");
    ctx->relabel_spin_limit = (unsigned)value;
    return DCI_OK;
  }
  if (option == DCI_OPT_TEST_RELABEL_FIRST_TICKET) {
    if (value < 0 || value > 65536)
      return dci::fail(ctx, DCI_ERR_INVALID_ARG, "DCI_OPT_TEST_RELABEL_FIRST_TICKET takes 0 .. 65536, not %lld", (long long)value);
    if (value != 0 && ctx->relabel_spin_limit > 65536)
      return dci::fail(ctx, DCI_ERR_INVALID_ARG, "lower DCI_OPT_RELABEL_SPIN_LIMIT to 65536 or less before switching the first-ticket test hook on");
    ctx->test_first_ticket = (unsigned)value;
    return DCI_OK;
  }
  return dci::fail(ctx, DCI_ERR_INVALID_ARG, "unknown option %d", option);
}

int32_t dci_blocks_bounds(int64_t num_nodes, int64_t n_seeds, const int32_t* fanouts, int32_t n_hops,
                          int64_t* cap_nodes, int64_t* cap_edges) {
  if (num_nodes < 1 || n_seeds < 0 || !fanouts || n_hops < 1 || n_hops > DCI_MAX_HOPS || !cap_nodes || !cap_edges)
    return DCI_ERR_INVALID_ARG;
  const int64_t limit = (int64_t)1 << 31;
  cap_nodes[0] = n_seeds;
  for (int32_t h = 0; h < n_hops; ++h) {
    if (fanouts[h] < 1 || fanouts[h] > DCI_MAX_FANOUT) return DCI_ERR_INVALID_ARG;
    if (cap_nodes[h] >= limit) return DCI_ERR_UNSUPPORTED;
    cap_edges[h] = cap_nodes[h] * fanouts[h];
    int64_t grown = cap_nodes[h] * (1 + (int64_t)fanouts[h]);
    int64_t all = num_nodes + n_seeds;
    cap_nodes[h + 1] = grown < all ? grown : all;
    if (cap_edges[h] >= limit || cap_nodes[h + 1] >= limit) return DCI_ERR_UNSUPPORTED;
  }
  return DCI_OK;
}

}  // extern "C"
