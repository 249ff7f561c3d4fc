// Measurement hook for the co-location experiment (paper section 3.5, "Physical Co-Location and
// Spatial Multiplexing": stages with dissimilar resource demands share one device): a synthetic
// memory-bound neighbour for the encoder.  It streams a large buffer once per launch, 16 bytes
// per lane and load, and keeps one sum per block -- the access pattern of a decode step reading
// its weights and KV cache, with next to no arithmetic.  Not part of the Encode path.
#include "../../include/epd_encode.h"
#include "epd_internal.h"

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

// ---- matrix-core rate on register-resident operands: no memory traffic at all, so what it
// measures is the matrix pipes under the chip's power limit.  Every wave cycles through eight
// A and eight B fragments (both operands change with every instruction) and four accumulators.
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

__device__ inline bf16x8 probe_fragment(uint32_t& s, bool zero) {
  union { bf16x8 v; uint32_t w[4]; } u;
  for (int i = 0; i < 4; ++i) {
    s = s * 1664525u + 1013904223u;
    // two bf16 values of magnitude [0.5, 1) with random sign and mantissa
    u.w[i] = zero ? 0u : (((s & 0x807f) | 0x3f00) | ((((s >> 16) & 0x807f) | 0x3f00) << 16));
  }
  return u.v;
}

template <int SHAPE>   // 0: v_mfma_f32_32x32x16_bf16, 1: v_mfma_f32_16x16x32_bf16
__global__ __launch_bounds__(512) void mfma_rate_kernel(int iters, int zero, float* out) {
  uint32_t seed = threadIdx.x * 9781u + blockIdx.x * 7919u + 1u;
  bf16x8 a[8], b[8];
  for (int i = 0; i < 8; ++i) { a[i] = probe_fragment(seed, zero != 0); b[i] = probe_fragment(seed, zero != 0); }
  float s = 0.f;
  if constexpr (SHAPE == 0) {
    f32x16 acc[4];
    for (int i = 0; i < 4; ++i) for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < 32; ++i) acc[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i & 7], b[(i * 3 + 1) & 7], acc[i & 3], 0, 0, 0);
    }
    for (int i = 0; i < 4; ++i) for (int v = 0; v < 16; ++v) s += acc[i][v];
  } else {
    f32x4 acc[4];
    for (int i = 0; i < 4; ++i) for (int v = 0; v < 4; ++v) acc[i][v] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < 64; ++i) acc[i & 3] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i & 7], b[(i * 3 + 1) & 7], acc[i & 3], 0, 0, 0);
    }
    for (int i = 0; i < 4; ++i) for (int v = 0; v < 4; ++v) s += acc[i][v];
  }
  out[blockIdx.x * 512 + threadIdx.x] = s;
}

}  // namespace

// 256 blocks of 8 waves (two per SIMD on a 256-CU chip).  One launch executes
// 256 * 8 * iters * 32 * 32768 flops: a 32x32x16 instruction is 2 * 32 * 32 * 16 = 32768 flops and a
// wave issues 32 of them per iteration (or 64 of the half-sized 16x16x32).
extern "C" epd_status epd_probe_mfma_rate(int32_t shape, int32_t zero_operands, int32_t iters, float* device_out,
                                          double* flops_per_launch, void* stream) {
  if ((shape != 0 && shape != 1) || iters <= 0 || !device_out) return EPD_ERR_INVALID_ARG;
  if (shape == 0) hipLaunchKernelGGL(mfma_rate_kernel<0>, dim3(256), dim3(512), 0, (hipStream_t)stream, iters, zero_operands, device_out);
  else hipLaunchKernelGGL(mfma_rate_kernel<1>, dim3(256), dim3(512), 0, (hipStream_t)stream, iters, zero_operands, device_out);
  if (flops_per_launch) *flops_per_launch = 256.0 * 8.0 * (double)iters * 32.0 * 32768.0;
  return hipGetLastError() == hipSuccess ? EPD_OK : EPD_ERR_HIP;
}

extern "C" epd_status epd_probe_stream_read(const void* device_buf, uint64_t bytes, float* device_out, int32_t blocks,
                                            void* stream) {
  if (!device_buf || !device_out || blocks <= 0 || blocks > 65536 || bytes < 16 || ((uintptr_t)device_buf & 15))
    return EPD_ERR_INVALID_ARG;
  hipLaunchKernelGGL(stream_read_kernel, dim3(blocks), dim3(kThreads), 0, (hipStream_t)stream, (const uint4*)device_buf,
                     bytes / 16, device_out);
  return hipGetLastError() == hipSuccess ? EPD_OK : EPD_ERR_HIP;
}

// Host only: the tiling launch_gemm_bf16 chooses for an M x N x K GEMM (see plan_gemm_bf16).
extern "C" epd_status epd_probe_gemm_plan(int32_t M, int32_t N, int32_t K, int32_t epilogue, int32_t qk_cols, int32_t compute_units,
                                          int32_t* tile_rows, int32_t* tile_cols, int32_t* body_rows) {
  if (M <= 0 || N <= 0 || K <= 0 || epilogue < 0 || epilogue > 3 || !tile_rows || !tile_cols || !body_rows ||
      (epilogue == epd::EPI_QKV && (qk_cols <= 0 || qk_cols > N)))
    return EPD_ERR_INVALID_ARG;
  epd::GemmArgs g{};
  g.M = M; g.N = N; g.K = K;
  g.epilogue = epilogue;
  g.qk_cols = epilogue == epd::EPI_QKV ? qk_cols : 0;
  int tr = 0, tc = 0, br = 0;
  epd::plan_gemm_bf16(g, compute_units, &tr, &tc, &br);
  *tile_rows = tr; *tile_cols = tc; *body_rows = br;
  return EPD_OK;
}
