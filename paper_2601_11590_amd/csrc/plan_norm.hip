// Per-call plan kernels, the fused LayerNorm / RMSNorm kernel and the create-time weight
// reordering of the Encode-stage library (ViT forward, paper section 3.1, Eq. 1).
//
// All of these are bound by memory traffic, not arithmetic: they use wide coalesced
// accesses and wave-level (64 lane) reductions, no matrix cores.
#include "epd_internal.h"

namespace epd {

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;

// ------------------------------------------------------------------------------ plan
__device__ __forceinline__ int upper_item(const int32_t* off, int n, int x) {
  // largest i in [0, n) with off[i] <= x   (off[0] = 0, off increasing)
  int lo = 0, hi = n;
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (off[mid] <= x) lo = mid; else hi = mid;
  }
  return lo;
}

// One thread per token: rotary table row and the token's column in the transposed V buffer.
__global__ __launch_bounds__(256) void plan_tokens_kernel(PlanArgs p) {
  int tok = blockIdx.x * blockDim.x + threadIdx.x;
  if (tok >= p.T) return;
  if (p.pairs > 0) {
    int it = upper_item(p.item_tok_off, p.num_items, tok);
    int local = tok - p.item_tok_off[it];
    int h = p.grid_thw[it * 3 + 1], w = p.grid_thw[it * 3 + 2];
    int coord[3];
    coord[0] = local / (h * w);
    int rem = local - coord[0] * h * w;
    coord[1] = rem / w;
    coord[2] = rem - coord[1] * w;
    for (int q = 0; q < p.pairs; ++q) {
      double ang = (double)coord[p.pair_axis[q]] * p.pair_freq[q];
      double sn, cs;
      sincos(ang, &sn, &cs);
      p.rot[(size_t)tok * p.pairs + q] = make_float2((float)cs, (float)sn);
    }
  }
  if (p.vcol) {
    int sg = upper_item(p.cu, p.num_segments, tok);
    p.vcol[tok] = p.pcu[sg] + (tok - p.cu[sg]);
  }
}

// One thread per merged token: the merge*merge source tokens, window rows then columns.
__global__ __launch_bounds__(256) void plan_merge_kernel(PlanArgs p) {
  int mt = blockIdx.x * blockDim.x + threadIdx.x;
  if (mt >= p.Tm) return;
  int it = upper_item(p.item_mrg_off, p.num_items, mt);
  int local = mt - p.item_mrg_off[it];
  int m = p.merge;
  int h = p.grid_thw[it * 3 + 1], w = p.grid_thw[it * 3 + 2];
  int hm = h / m, wm = w / m;
  int ti = local / (hm * wm);
  int rem = local - ti * hm * wm;
  int i = rem / wm, j = rem - i * wm;
  int base = p.item_tok_off[it] + ti * h * w;
  for (int di = 0; di < m; ++di)
    for (int dj = 0; dj < m; ++dj)
      p.merge_idx[(size_t)mt * m * m + di * m + dj] = base + (m * i + di) * w + m * j + dj;
}

// Clear the columns of the transposed V buffer between a segment's end and the next
// segment's (aligned) start: attention multiplies them by exact zeros, so they must be finite.
__global__ __launch_bounds__(128) void plan_clear_vt_pad_kernel(PlanArgs p) {
  int sg = blockIdx.x;
  int row = blockIdx.y;
  int len = p.cu[sg + 1] - p.cu[sg];
  int c0 = p.pcu[sg] + len, c1 = p.pcu[sg + 1];
  uint16_t* vt = (uint16_t*)p.vt + (size_t)row * p.vt_stride;
  for (int c = c0 + threadIdx.x; c < c1; c += blockDim.x) vt[c] = 0;
}

void launch_plan(const PlanArgs& p, hipStream_t s) {
  if (p.T > 0 && (p.pairs > 0 || p.vcol))
    hipLaunchKernelGGL(plan_tokens_kernel, dim3((p.T + 255) / 256), dim3(256), 0, s, p);
  if (p.Tm > 0 && p.merge > 1)
    hipLaunchKernelGGL(plan_merge_kernel, dim3((p.Tm + 255) / 256), dim3(256), 0, s, p);
  if (p.vt && p.num_segments > 0)
    hipLaunchKernelGGL(plan_clear_vt_pad_kernel, dim3(p.num_segments, p.hidden), dim3(128), 0, s, p);
}

// ------------------------------------------------------------------------------ norm
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}


template <typename T> __device__ __forceinline__ void ld_param4(const T* p, int i, float* o);
template <> __device__ __forceinline__ void ld_param4<float>(const float* p, int i, float* o) {
  const float4 v = *(const float4*)(p + i);
  o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
}
template <> __device__ __forceinline__ void ld_param4<__bf16>(const __bf16* p, int i, float* o) {
  const uint2 v = *(const uint2*)(p + i);
  o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xffff0000u);
  o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xffff0000u);
}

// One 64-lane wave per token row; the row is held in registers (NV float4 per lane) between
// the statistics pass and the scaling pass, so HBM sees one read and one write per element.
// LayerNorm uses the two-pass mean / centred variance form (biased variance).
template <typename PT, typename OT, int NV>
__global__ __launch_bounds__(256) void norm_kernel(const float* __restrict__ x, const PT* __restrict__ gamma,
                                                   const PT* __restrict__ beta, OT* __restrict__ out,
                                                   int T, int D, float eps, int rms) {
  int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  int lane = threadIdx.x & 63;
  if (row >= T) return;
  const float* xr = x + (size_t)row * D;
  float4 v[NV];
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    int c = (i * 64 + lane) * 4;
    v[i] = (c < D) ? *(const float4*)(xr + c) : make_float4(0.f, 0.f, 0.f, 0.f);
    sum += (v[i].x + v[i].y) + (v[i].z + v[i].w);
  }
  float mean = 0.f;
  if (!rms) mean = wave_sum(sum) / (float)D;
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    int c = (i * 64 + lane) * 4;
    if (c < D) {
      float a = v[i].x - mean, b = v[i].y - mean, cc = v[i].z - mean, d = v[i].w - mean;
      sq += (a * a + b * b) + (cc * cc + d * d);
    }
  }
  float rstd = 1.0f / sqrtf(wave_sum(sq) / (float)D + eps);   // correctly rounded, once per row
  OT* orow = out + (size_t)row * D;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    int c = (i * 64 + lane) * 4;
    if (c < D) {
      float y[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
      // the four gains (and shifts) of the chunk come in one load each (c is a multiple of 4)
      float g4[4], b4[4] = {0.f, 0.f, 0.f, 0.f};
      ld_param4(gamma, c, g4);
      if (beta) ld_param4(beta, c, b4);
#pragma unroll
      for (int e = 0; e < 4; ++e) y[e] = (y[e] - mean) * rstd * g4[e] + b4[e];
      if constexpr (sizeof(OT) == 4) {
        *(float4*)((float*)orow + c) = make_float4(y[0], y[1], y[2], y[3]);
      } else {
        bf16x2_t lo, hi;
        lo[0] = (__bf16)y[0]; lo[1] = (__bf16)y[1];
        hi[0] = (__bf16)y[2]; hi[1] = (__bf16)y[3];
        uint2 pk;
        pk.x = *(uint32_t*)&lo; pk.y = *(uint32_t*)&hi;
        *(uint2*)((__bf16*)orow + c) = pk;
      }
    }
  }
}

template <typename PT, typename OT>
static void norm_dispatch(const float* x, const void* g, const void* b, void* out, int T, int D,
                          float eps, bool rms, hipStream_t s) {
  dim3 grid((T + 3) / 4), block(256);
  int nv = (D + 255) / 256;
#define EPD_NORM_CASE(N)                                                                      \
  hipLaunchKernelGGL((norm_kernel<PT, OT, N>), grid, block, 0, s, x, (const PT*)g, (const PT*)b, \
                     (OT*)out, T, D, eps, rms ? 1 : 0)
  if (nv <= 1) EPD_NORM_CASE(1);
  else if (nv <= 2) EPD_NORM_CASE(2);
  else if (nv <= 4) EPD_NORM_CASE(4);
  else if (nv <= 5) EPD_NORM_CASE(5);
  else if (nv <= 8) EPD_NORM_CASE(8);
  else if (nv <= 13) EPD_NORM_CASE(13);
  else if (nv <= 16) EPD_NORM_CASE(16);
  else EPD_NORM_CASE(32);   // D <= 8192 (checked at create)
#undef EPD_NORM_CASE
}

void launch_norm(const float* x, const void* gamma, const void* beta, void* out, int T, int D,
                 float eps, bool rms, bool bf16, hipStream_t s) {
  if (T <= 0) return;
  if (bf16) norm_dispatch<__bf16, __bf16>(x, gamma, beta, out, T, D, eps, rms, s);
  else norm_dispatch<float, float>(x, gamma, beta, out, T, D, eps, rms, s);
}

// ------------------------------------------------------------------------------ create-time reorder
// Rows of the fused QKV weight are reordered inside every Q and K head so that the two
// members (p, p + d/2) of rotary pair p become neighbours (2p, 2p + 1).  Q.K^T is
// unchanged by a permutation applied to both, and the GEMM epilogue can then rotate a pair
// without leaving the lane that owns it.  V rows are copied as they are.
template <typename T>
__global__ __launch_bounds__(256) void permute_qkv_kernel(const T* __restrict__ sw, const T* __restrict__ sb,
                                                          T* __restrict__ dw, T* __restrict__ db,
                                                          int D, int hd) {
  int drow = blockIdx.x;     // destination row in [0, 3D)
  int srow = drow;
  if (drow < 2 * D) {
    int head0 = (drow / hd) * hd;
    int c = drow - head0;
    srow = head0 + (c >> 1) + (c & 1) * (hd >> 1);
  }
  const T* s = sw + (size_t)srow * D;
  T* d = dw + (size_t)drow * D;
  for (int i = threadIdx.x; i < D; i += blockDim.x) d[i] = s[i];
  if (sb && threadIdx.x == 0) db[drow] = sb[srow];
}

void launch_permute_qkv(const void* src_w, const void* src_b, void* dst_w, void* dst_b, int hidden,
                        int num_heads, int head_dim, int elem_bytes, hipStream_t s) {
  (void)num_heads;
  if (elem_bytes == 4)
    hipLaunchKernelGGL(permute_qkv_kernel<float>, dim3(3 * hidden), dim3(256), 0, s, (const float*)src_w,
                       (const float*)src_b, (float*)dst_w, (float*)dst_b, hidden, head_dim);
  else
    hipLaunchKernelGGL(permute_qkv_kernel<uint16_t>, dim3(3 * hidden), dim3(256), 0, s, (const uint16_t*)src_w,
                       (const uint16_t*)src_b, (uint16_t*)dst_w, (uint16_t*)dst_b, hidden, head_dim);
}

// ---------------------------------------------------------------- gamma folding (create time)
__global__ __launch_bounds__(256) void fold_gamma_kernel(uint16_t* __restrict__ w, const uint16_t* __restrict__ gamma,
                                                         long total, int K) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int k = (int)(i % K);
  const float v = __uint_as_float((uint32_t)w[i] << 16) * __uint_as_float((uint32_t)gamma[k] << 16);
  __bf16 r = (__bf16)v;   // round to nearest even
  w[i] = *(uint16_t*)&r;
}

void launch_fold_gamma(void* w, const void* gamma, int N, int K, hipStream_t s) {
  const long total = (long)N * K;
  hipLaunchKernelGGL(fold_gamma_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, (uint16_t*)w,
                     (const uint16_t*)gamma, total, K);
}

}  // namespace epd
