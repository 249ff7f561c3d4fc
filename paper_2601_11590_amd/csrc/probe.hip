// Measurement hook for the co-location experiment (paper section 3.5, "Physical Co-Location and
// Spatial Multiplexing": stages with dissimilar resource demands share one device): a synthetic
// memory-bound neighbour for the encoder.  It streams a large buffer once per launch, 16 bytes
// per lane and load, and keeps one sum per block -- the access pattern of a decode step reading
// its weights and KV cache, with next to no arithmetic.  Not part of the Encode path.
#include "../../include/epd_encode.h"

#include <hip/hip_runtime.h>

namespace {

constexpr int kThreads = 256;

__global__ __launch_bounds__(kThreads) void stream_read_kernel(const uint4* __restrict__ buf, uint64_t n16, float* __restrict__ out) {
  uint32_t acc = 0;
  // four independent 16-byte loads per lane and trip keep enough bytes in flight per CU
  const uint64_t stride = (uint64_t)gridDim.x * kThreads;
  uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const uint4 a = buf[i], b = buf[i + stride], c = buf[i + 2 * stride], d = buf[i + 3 * stride];
    acc += (a.x ^ a.y) + (a.z ^ a.w) + (b.x ^ b.y) + (b.z ^ b.w) + (c.x ^ c.y) + (c.z ^ c.w) + (d.x ^ d.y) + (d.z ^ d.w);
  }
  for (; i < n16; i += stride) {
    const uint4 a = buf[i];
    acc += (a.x ^ a.y) + (a.z ^ a.w);
  }
  __shared__ uint32_t part[kThreads];
  part[threadIdx.x] = acc;
  __syncthreads();
  for (int s = kThreads / 2; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) part[threadIdx.x] += part[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[blockIdx.x] = (float)(part[0] & 0xffffff);
}

}  // namespace

extern "C" epd_status epd_probe_stream_read(const void* device_buf, uint64_t bytes, float* device_out, int32_t blocks,
                                            void* stream) {
  if (!device_buf || !device_out || blocks <= 0 || blocks > 65536 || bytes < 16 || ((uintptr_t)device_buf & 15))
    return EPD_ERR_INVALID_ARG;
  hipLaunchKernelGGL(stream_read_kernel, dim3(blocks), dim3(kThreads), 0, (hipStream_t)stream, (const uint4*)device_buf,
                     bytes / 16, device_out);
  return hipGetLastError() == hipSuccess ? EPD_OK : EPD_ERR_HIP;
}
