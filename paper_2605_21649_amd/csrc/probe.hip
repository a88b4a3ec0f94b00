// Streaming-read probe: what a kernel that does nothing but read pages of a buffer achieves on the GPU at hand.
// It is the measured ceiling the HBM-bound kernels of the library are compared with (next to the published
// peak).  One wavefront reads four pages of `page_bytes` bytes with 16-byte loads, all requested before any is
// consumed; the page numbers come from a list (a permutation for the gather pattern of the decode, the identity for
// a linear stream) through wave-uniform scalar loads.  Two optional features give the probe the memory behaviour
// of the decode's score pass without its arithmetic: a second dependent lookup per page (page list -> block
// table) and 256 bytes of output per wavefront (the scores of 64 tokens).
#include "ekv_device.h"
#include "ekv_internal.h"

namespace ekv {

constexpr int kProbePagesPerWave = 4;

template <int KB>     // KiB per page
__global__ __launch_bounds__(256) void probe_read_kernel(const uint4* __restrict__ base, const int32_t* page_ids,
                                                         const int32_t* lookup, int n_pages, float* out,
                                                         uint32_t* sink) {
  constexpr int PPW = kProbePagesPerWave;
  const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wave = blockIdx.x * 4 + w;
  const int p0 = wave * PPW;
  if (p0 >= n_pages) return;
  int ids[PPW];
#pragma unroll
  for (int i = 0; i < PPW; ++i) ids[i] = uniform_load(page_ids + min(p0 + i, n_pages - 1));
  if (lookup != nullptr) {
#pragma unroll
    for (int i = 0; i < PPW; ++i) ids[i] = uniform_load(lookup + ids[i]);
  }
  uint4 v[PPW][KB];
#pragma unroll
  for (int i = 0; i < PPW; ++i)
#pragma unroll
    for (int s = 0; s < KB; ++s) v[i][s] = base[(size_t)ids[i] * (KB * 64) + s * 64 + lane];
  uint32_t acc = 0;
#pragma unroll
  for (int i = 0; i < PPW; ++i)
#pragma unroll
    for (int s = 0; s < KB; ++s) acc ^= v[i][s].x ^ v[i][s].y ^ v[i][s].z ^ v[i][s].w;
  if (acc == 0x9e3779b9u) sink[0] = acc;       // keeps the loads alive; practically never taken
  if (out != nullptr) out[(size_t)wave * 64 + lane] = __uint_as_float(acc);
}

void launch_probe_read(const void* base, const int32_t* page_ids, const int32_t* lookup, int n_pages, int page_bytes,
                       float* out, uint32_t* sink, hipStream_t st) {
  const int waves = (n_pages + kProbePagesPerWave - 1) / kProbePagesPerWave;
  dim3 grid((waves + 3) / 4), block(256);
  if (page_bytes == 4096)
    hipLaunchKernelGGL((probe_read_kernel<4>), grid, block, 0, st, (const uint4*)base, page_ids, lookup, n_pages, out, sink);
  else
    hipLaunchKernelGGL((probe_read_kernel<8>), grid, block, 0, st, (const uint4*)base, page_ids, lookup, n_pages, out, sink);
}

// Hand-off probe: what it costs to pass data between workgroups INSIDE one launch (the alternative to a kernel
// boundary when two dependent stages are to be fused).  Every workgroup writes 4 KiB; then, by `mode`:
//   0  nothing more (the reference);
//   1  device-scope fence, an acquire-release counter, the last workgroup to arrive fences and reads 8 KiB that
//      other workgroups wrote (the classic last-arriver reduction);
//   2  the same without fences: the data is written with device-scope atomic stores (write-through), the counter
//      is relaxed, the last arriver reads with device-scope atomic loads.
// The counter is left at zero for the next launch.
__global__ __launch_bounds__(256) void probe_handoff_kernel(float* data, uint32_t* counter, float* out, int mode) {
  __shared__ bool last;
  constexpr int kWords = 1024;
  float* mine = data + (size_t)blockIdx.x * kWords;
  for (int i = threadIdx.x; i < kWords; i += 256) {
    const float v = (float)(blockIdx.x + i);
    if (mode == 2) __hip_atomic_store(mine + i, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else mine[i] = v;
  }
  if (mode == 0) return;
  if (mode == 1) __threadfence();
  __syncthreads();
  if (threadIdx.x == 0) {
    const uint32_t old = __hip_atomic_fetch_add(counter, 1u, mode == 1 ? __ATOMIC_ACQ_REL : __ATOMIC_RELAXED,
                                                __HIP_MEMORY_SCOPE_AGENT);
    last = old == gridDim.x - 1;
  }
  __syncthreads();
  if (!last) return;
  if (mode == 1) __threadfence();
  const size_t n_all = (size_t)gridDim.x * kWords;
  float s = 0.f;
  for (int i = threadIdx.x; i < 2048; i += 256) {
    const float* p = data + ((size_t)i * 257) % n_all;
    s += mode == 2 ? __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : *p;
  }
  s = wave_sum(s);
  if ((threadIdx.x & 63) == 0) atomicAdd(out, s);
  if (threadIdx.x == 0) *counter = 0;
}

void launch_probe_handoff(float* data, uint32_t* counter, float* out, int n_workgroups, int mode, hipStream_t st) {
  hipLaunchKernelGGL(probe_handoff_kernel, dim3(n_workgroups), dim3(256), 0, st, data, counter, out, mode);
}

}  // namespace ekv
