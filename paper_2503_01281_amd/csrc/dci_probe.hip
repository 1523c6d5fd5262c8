// Memory-rate probes: the denominators that the access-bound kernels of the path are measured
// against (streaming and random reads of HBM, and of pinned host memory through the host link).
// They read, fold what they read into one word per workgroup so that no load can be dropped, and
// are timed with events on the context's stream.  Nothing of the method's arithmetic is here.
#include "dci_internal.h"

namespace dci {

constexpr int kProbeBlock = 256;

__device__ __forceinline__ unsigned long long probe_mix(unsigned long long z) {
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// Streaming read: consecutive lanes on consecutive 16-byte words, four loads in flight per lane.
__global__ __launch_bounds__(kProbeBlock) void k_probe_stream(const uint4* __restrict__ p, size_t n16,
                                                              unsigned long long* __restrict__ sink) {
  unsigned acc = 0;
  const size_t stride = (size_t)gridDim.x * kProbeBlock;
  size_t i = blockIdx.x * (size_t)kProbeBlock + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const uint4 a = p[i], b = p[i + stride], c = p[i + 2 * stride], d = p[i + 3 * stride];
    acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
  }
  for (; i < n16; i += stride) {
    const uint4 a = p[i];
    acc ^= a.x ^ a.y ^ a.z ^ a.w;
  }
  if (acc == 0x9E3779B9u) sink[blockIdx.x] = acc;  // practically never true; keeps the loads alive
}

// Random reads of aligned granules.  LANES lanes share one granule (LANES * W bytes, W = bytes per
// lane: 8 or 16); access a of the launch reads granule hash(seed, a) mod n_granules; every lane
// group issues `kInFlight` independent accesses before it uses any of them.
// order: 0 = the lanes of a group take the granule's words in lane order,
//        1 = in a scrambled order (same bytes, the lanes of one line are still adjacent lanes),
//        2 = the 64 lanes of a wavefront are dealt out so that the lanes of one granule are
//            LANES-strided, i.e. never adjacent (what scattered slots of one list look like).
template <int W, int LANES>
__global__ __launch_bounds__(kProbeBlock) void k_probe_random(const char* __restrict__ p,
                                                              unsigned long long n_granules, long long n_access,
                                                              unsigned long long seed, int order,
                                                              unsigned long long* __restrict__ sink) {
  constexpr int kInFlight = 4;
  constexpr int kGroupsPerBlock = kProbeBlock / LANES;
  constexpr int kGroupsPerWave = kWave / LANES;
  const int lane = (int)threadIdx.x & (kWave - 1);
  int grp_in_wave, word;
  if (order == 2) {
    grp_in_wave = lane % kGroupsPerWave;
    word = lane / kGroupsPerWave;
  } else {
    grp_in_wave = lane / LANES;
    word = lane % LANES;
    if (order == 1) word = (word * 5 + 3) % LANES;  // a fixed permutation of 0..LANES-1 (LANES is a power of two)
  }
  const long long grp = (long long)blockIdx.x * kGroupsPerBlock + ((int)threadIdx.x / kWave) * kGroupsPerWave + grp_in_wave;
  const long long n_groups = (long long)gridDim.x * kGroupsPerBlock;
  unsigned long long acc = 0;
  for (long long a = grp; a < n_access; a += n_groups * kInFlight) {
    unsigned long long v[kInFlight];
#pragma unroll
    for (int u = 0; u < kInFlight; ++u) {
      const long long idx = a + (long long)u * n_groups;
      if (idx < n_access) {
        const unsigned long long gidx = probe_mix(seed ^ probe_mix((unsigned long long)idx)) % n_granules;
        const char* at = p + gidx * (unsigned long long)(W * LANES) + (unsigned)word * W;
        if (W == 16) {
          const uint4 q = *reinterpret_cast<const uint4*>(at);
          v[u] = (unsigned long long)(q.x ^ q.z) | ((unsigned long long)(q.y ^ q.w) << 32);
        } else {
          v[u] = *reinterpret_cast<const unsigned long long*>(at);
        }
      } else {
        v[u] = 0;
      }
    }
#pragma unroll
    for (int u = 0; u < kInFlight; ++u) acc ^= v[u];
  }
  if (acc == 0x9E3779B97F4A7C15ull) sink[blockIdx.x] = acc;
}

template <int W, int LANES>
static void launch_random(dci_ctx* ctx, int grid, const void* p, uint64_t bytes, int64_t n_access, uint64_t seed,
                          int order, uint64_t* sink) {
  hipLaunchKernelGGL((k_probe_random<W, LANES>), dim3(grid), dim3(kProbeBlock), 0, ctx->stream,
                     reinterpret_cast<const char*>(p), (unsigned long long)(bytes / (uint64_t)(W * LANES)),
                     (long long)n_access, (unsigned long long)seed, order,
                     reinterpret_cast<unsigned long long*>(sink));
}

}  // namespace dci

using namespace dci;

extern "C" int32_t dci_probe_read(dci_ctx* ctx, const void* mem, uint64_t bytes, int32_t granule, int32_t order,
                                  int64_t n_access, int32_t workgroups, uint64_t seed, uint64_t* sink,
                                  float* ms) {
  if (!ctx) return DCI_ERR_INVALID_ARG;
  if (!mem || !sink || !ms || bytes < 4096 || (reinterpret_cast<uintptr_t>(mem) & 255) || order < 0 || order > 2 ||
      workgroups < 1 || workgroups > 65536)
    return fail(ctx, DCI_ERR_INVALID_ARG, "probe_read: null / unaligned / tiny region, or order / workgroups out of range");
  if (granule != 0 && n_access < 1) return fail(ctx, DCI_ERR_INVALID_ARG, "probe_read: n_access < 1");
  DCI_HIP(ctx, hipEventRecord(ctx->ev[0], ctx->stream));
  switch (granule) {
    case 0:
      hipLaunchKernelGGL(k_probe_stream, dim3(workgroups), dim3(kProbeBlock), 0, ctx->stream,
                         reinterpret_cast<const uint4*>(mem), (size_t)(bytes / 16),
                         reinterpret_cast<unsigned long long*>(sink));
      break;
    case 8: launch_random<8, 1>(ctx, workgroups, mem, bytes, n_access, seed, order, sink); break;
    case 16: launch_random<16, 1>(ctx, workgroups, mem, bytes, n_access, seed, order, sink); break;
    case 32: launch_random<16, 2>(ctx, workgroups, mem, bytes, n_access, seed, order, sink); break;
    case 64: launch_random<16, 4>(ctx, workgroups, mem, bytes, n_access, seed, order, sink); break;
    case 128: launch_random<16, 8>(ctx, workgroups, mem, bytes, n_access, seed, order, sink); break;
    case 256: launch_random<16, 16>(ctx, workgroups, mem, bytes, n_access, seed, order, sink); break;
    case 512: launch_random<16, 32>(ctx, workgroups, mem, bytes, n_access, seed, order, sink); break;
    case -64: launch_random<8, 8>(ctx, workgroups, mem, bytes, n_access, seed, order, sink); break;
    default: return fail(ctx, DCI_ERR_INVALID_ARG, "probe_read: granule must be 0, 8, 16, 32, 64, 128, 256, 512 or -64");
  }
  DCI_LAUNCH_CHECK(ctx);
  DCI_HIP(ctx, hipEventRecord(ctx->ev[1], ctx->stream));
  DCI_HIP(ctx, hipEventSynchronize(ctx->ev[1]));
  DCI_HIP(ctx, hipEventElapsedTime(ms, ctx->ev[0], ctx->ev[1]));
  return DCI_OK;
}
