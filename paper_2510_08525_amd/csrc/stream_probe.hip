// Measurement aid: a plain streaming read of a device buffer, for a measured ceiling beside the
// nominal HBM peak.  Same access shape as the decode kernel's K/V stream (each wavefront reads
// 16 KiB blocks with 128-bit non-temporal loads, a workgroup owns one contiguous range) and no
// arithmetic beyond an xor that keeps the loads alive.
#include "rlkv_internal.h"

namespace rlkv {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(kBlock) void stream_read_kernel(const char* __restrict__ buf, int64_t n_blocks,
                                                             uint32_t* __restrict__ sink) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int64_t per_wg = (n_blocks + gridDim.x - 1) / gridDim.x;
  const int64_t first = (int64_t)blockIdx.x * per_wg;
  const int64_t last = first + per_wg < n_blocks ? first + per_wg : n_blocks;
  u32x4 acc = u32x4{0, 0, 0, 0};
  for (int64_t t = first + wave; t < last; t += 4) {
    const char* p = buf + t * kTileBytes + lane * 16;
    u32x4 r[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) r[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p + i * 1024));
#pragma unroll
    for (int i = 0; i < 16; ++i) acc ^= r[i];
  }
  const uint32_t x = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
  if (x == 0x9e3779b9u) sink[0] = x;      // practically never; the compiler cannot drop the loads
}

}  // namespace

hipError_t launch_stream_read(const void* buf, size_t bytes, void* sink, int workgroups, hipStream_t stream) {
  const int64_t n_blocks = (int64_t)(bytes / kTileBytes);
  if (n_blocks == 0) return hipSuccess;
  hipLaunchKernelGGL(stream_read_kernel, dim3(workgroups), dim3(kBlock), 0, stream, (const char*)buf, n_blocks,
                     (uint32_t*)sink);
  return hipGetLastError();
}

}  // namespace rlkv
