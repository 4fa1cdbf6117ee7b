// Measurement aids (no part of the method): bare kernels that move known numbers of bytes, so that a
// benchmark can quote the shrink / expand kernels against what this GPU's memory system delivers to
// the simplest possible code with the same mix of accesses, and a single large pinned host -> device
// copy as the roof of the adapter loads.  See include/plora.h (plora_probe_*).
#include "../../include/plora.h"

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// Every workgroup walks over tiles of the two buffers in turn, grid-stride.  For a tile it first requests
// its piece of `y` (y_tile bytes, at most 16 bytes per thread and pass), then reads its piece of `w`
// (w_tile bytes) with streaming 16-byte loads, four in flight per thread, and finally writes the changed
// piece of y back with streaming stores: the order in which the expand kernels touch the rows of y of an
// item's tokens and the item's weights.  y_tile = 0 gives the plain streaming read.  What is read is
// folded into a value that is stored only if it has a bit pattern that does not occur, so the loads cannot
// be dropped.
__global__ __launch_bounds__(256) void k_probe(const uint8_t* __restrict__ w, uint64_t w_bytes, uint32_t w_tile,
                                                uint8_t* __restrict__ y, uint64_t y_bytes, uint32_t y_tile,
                                                uint32_t* __restrict__ sink) {
  const uint64_t n_tiles = w_bytes / w_tile;
  u32x4_t fold = {0u, 0u, 0u, 0u};
  for (uint64_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
    const uint8_t* wp = w + t * w_tile;
    uint8_t* yp = y_tile ? y + (t * y_tile) % y_bytes : nullptr;
    for (uint32_t yo = 0; yo < (y_tile ? y_tile : 1u); yo += 256u * 16u) {
      const uint32_t mine = yo + threadIdx.x * 16u;
      const bool has_y = y_tile && mine < y_tile;
      u32x4_t yq = {0u, 0u, 0u, 0u};
      if (has_y) yq = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(yp + mine));
      if (yo == 0) {  // the weights of the tile go with the first pass over y
        for (uint32_t o = threadIdx.x * 16u; o < w_tile; o += 256u * 16u * 4u) {
          u32x4_t q[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const uint32_t ou = o + (uint32_t)u * 256u * 16u;
            q[u] = ou < w_tile ? __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(wp + ou)) : fold;
          }
#pragma unroll
          for (int u = 0; u < 4; ++u) fold ^= q[u];
        }
      }
      if (has_y) {
        yq += fold.x & 1u;
        __builtin_nontemporal_store(yq, reinterpret_cast<u32x4_t*>(yp + mine));
      }
    }
  }
  if ((fold.x ^ fold.y ^ fold.z ^ fold.w) == 0x9e3779b9u && fold.x == 0x7f4a7c15u) sink[0] = fold.y;
}

int fail(hipError_t e) {
  (void)e;
  (void)hipGetLastError();
  return PLORA_ERR_HIP;
}

}  // namespace

extern "C" int plora_probe_stream(uint64_t w_bytes, uint64_t y_bytes, uint32_t w_tile, uint32_t y_tile, int32_t iters,
                                  plora_stream stream, double* ms_per_launch) {
  if (!ms_per_launch || iters < 1 || iters > 10000 || w_tile < 4096 || (w_tile & 4095) || (y_tile & 4095)) return PLORA_ERR_INVAL;
  if (w_bytes < w_tile || w_bytes % w_tile || w_bytes > ((uint64_t)1 << 36)) return PLORA_ERR_INVAL;
  if ((y_tile != 0) != (y_bytes != 0) || (y_tile && (y_bytes < y_tile || y_bytes % y_tile)) || y_bytes > ((uint64_t)1 << 36))
    return PLORA_ERR_INVAL;
  hipStream_t st = (hipStream_t)stream;
  uint8_t *w = nullptr, *y = nullptr;
  uint32_t* sink = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  hipError_t e = hipMalloc((void**)&w, w_bytes);
  if (e == hipSuccess && y_bytes) e = hipMalloc((void**)&y, y_bytes);
  if (e == hipSuccess) e = hipMalloc((void**)&sink, 256);
  if (e == hipSuccess) e = hipMemsetAsync(w, 0x3c, w_bytes, st);
  if (e == hipSuccess && y_bytes) e = hipMemsetAsync(y, 0x01, y_bytes, st);
  if (e == hipSuccess) e = hipEventCreate(&e0);
  if (e == hipSuccess) e = hipEventCreate(&e1);
  float ms = 0.f;
  if (e == hipSuccess) {
    // as many workgroups as stay resident together on 256 compute units (8 x 256 threads each)
    const unsigned grid = 256u * 8u;
    for (int it = 0; it < 3; ++it) hipLaunchKernelGGL(k_probe, dim3(grid), dim3(256), 0, st, w, w_bytes, w_tile, y, y_bytes, y_tile, sink);
    e = hipEventRecord(e0, st);
    for (int it = 0; it < iters; ++it) hipLaunchKernelGGL(k_probe, dim3(grid), dim3(256), 0, st, w, w_bytes, w_tile, y, y_bytes, y_tile, sink);
    if (e == hipSuccess) e = hipEventRecord(e1, st);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    if (e == hipSuccess) e = hipGetLastError();
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  }
  (void)hipStreamSynchronize(st);
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (w) (void)hipFree(w);
  if (y) (void)hipFree(y);
  if (sink) (void)hipFree(sink);
  if (e != hipSuccess) return fail(e);
  *ms_per_launch = (double)ms / iters;
  return PLORA_OK;
}

extern "C" int plora_probe_h2d(uint64_t bytes, int32_t iters, plora_stream stream, double* ms_per_copy) {
  if (!ms_per_copy || iters < 1 || iters > 1000 || bytes < 4096 || bytes > ((uint64_t)1 << 34)) return PLORA_ERR_INVAL;
  hipStream_t st = (hipStream_t)stream;
  void *h = nullptr, *d = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  hipError_t e = hipHostMalloc(&h, bytes, hipHostMallocDefault);
  if (e == hipSuccess) e = hipMalloc(&d, bytes);
  if (e == hipSuccess) e = hipEventCreate(&e0);
  if (e == hipSuccess) e = hipEventCreate(&e1);
  float ms = 0.f;
  if (e == hipSuccess) {
    for (uint64_t o = 0; o < bytes; o += 4096) ((volatile uint8_t*)h)[o] = (uint8_t)o;  // pages touched
    e = hipMemcpyAsync(d, h, bytes, hipMemcpyHostToDevice, st);  // warm-up
    if (e == hipSuccess) e = hipEventRecord(e0, st);
    for (int it = 0; it < iters && e == hipSuccess; ++it) e = hipMemcpyAsync(d, h, bytes, hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipEventRecord(e1, st);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  }
  (void)hipStreamSynchronize(st);
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (d) (void)hipFree(d);
  if (h) (void)hipHostFree(h);
  if (e != hipSuccess) return fail(e);
  *ms_per_copy = (double)ms / iters;
  return PLORA_OK;
}
