// fp32 kernels of the Encode-stage library (ViT forward, paper section 3.1, Eq. 1): the
// configuration whose storage type is fp32 must multiply and accumulate in true fp32, so
// these use the vector ALU (fused multiply-add), not the reduced-precision matrix paths.
// They serve the small fp32 configuration; throughput work goes into the bf16 kernels.
#include "epd_internal.h"

namespace epd {

// ------------------------------------------------------------------------------ GEMM
// 64 x 64 output tile per 256-thread block, K in steps of 16 through LDS; each thread owns a
// 4 x 4 block (rows ty*4.., columns tx*4..), so the two members of a rotary pair (adjacent
// columns after the create-time reorder) sit in the same thread.
constexpr int F32_BM = 64, F32_BN = 64, F32_BK = 16;

__device__ __forceinline__ float gelu_f32(float v, int act) {
  if (act == 0) return 0.5f * v * (1.0f + erff(v * 0.70710678118654752440f));
  float u = 0.79788456080286535588f * (v + 0.044715f * v * v * v);
  return 0.5f * v * (1.0f + tanhf(u));
}

__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmArgs g) {
  __shared__ float As[F32_BK][F32_BM + 4];
  __shared__ float Ws[F32_BK][F32_BN + 4];
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.y * F32_BM, n0 = blockIdx.x * F32_BN;
  const float* A = (const float*)g.A;
  const float* W = (const float*)g.W;

  // loader mapping: 64 rows x 16 k; thread loads 4 consecutive k of one row
  const int lrow = tid >> 2, lk = (tid & 3) * 4;
  const int am = m0 + lrow, wn = n0 + lrow;
  const int kc = g.gather ? g.K / g.gather_n : g.K;   // width of one gathered piece

  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

  for (int k0 = 0; k0 < g.K; k0 += F32_BK) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      int k = k0 + lk + e;
      float av = 0.f, wv = 0.f;
      if (k < g.K) {
        if (am < g.M) {
          if (g.gather) {
            int piece = k / kc;
            int src = g.gather[(size_t)am * g.gather_n + piece];
            av = A[(size_t)src * g.lda + (k - piece * kc)];
          } else {
            av = A[(size_t)am * g.lda + k];
          }
        }
        if (wn < g.N) wv = W[(size_t)wn * g.K + k];
      }
      As[lk + e][lrow] = av;
      Ws[lk + e][lrow] = wv;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < F32_BK; ++kk) {
      float a[4], w[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) w[j] = Ws[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], w[j], acc[i][j]);
    }
    __syncthreads();
  }

  const float* bias = (const float*)g.bias;
  float* out = (float*)g.out;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int m = m0 + ty * 4 + i;
    if (m >= g.M) continue;
    float v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int n = n0 + tx * 4 + j;
      v[j] = acc[i][j] + ((bias && n < g.N) ? bias[n] : 0.f);
    }
    if (g.epilogue == EPI_QKV && g.rot) {
#pragma unroll
      for (int j = 0; j < 4; j += 2) {
        int n = n0 + tx * 4 + j;          // even column; pair = (n, n + 1)
        if (n + 1 < g.N && n < g.qk_cols) {
          int pr = (n % g.head_dim) >> 1;
          float2 cs = g.rot[(size_t)m * g.rot_pairs + pr];
          float a = v[j], b = v[j + 1];
          v[j] = a * cs.x - b * cs.y;
          v[j + 1] = a * cs.y + b * cs.x;
        }
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int n = n0 + tx * 4 + j;
      if (n >= g.N) continue;
      if (g.epilogue == EPI_RESIDUAL) g.resid[(size_t)m * g.ldr + n] += v[j];
      else if (g.epilogue == EPI_GELU) out[(size_t)m * g.ldo + n] = gelu_f32(v[j], g.act);
      else out[(size_t)m * g.ldo + n] = v[j];
    }
  }
}

void launch_gemm_f32(const GemmArgs& g, hipStream_t s) {
  if (g.M <= 0 || g.N <= 0) return;
  dim3 grid((g.N + F32_BN - 1) / F32_BN, (g.M + F32_BM - 1) / F32_BM);
  hipLaunchKernelGGL(gemm_f32_kernel, grid, dim3(256), 0, s, g);
}

// ------------------------------------------------------------------------------ attention
// One thread per query row (64 rows per work item), keys / values staged through LDS in
// tiles of 32 rows and read as broadcasts; running maximum / sum softmax in fp32 with expf.
constexpr int F32_BQ = 64, F32_BKV = 32;

template <int DH>
__global__ __launch_bounds__(64) void attn_f32_kernel(AttnArgs a) {
  __shared__ float Ks[F32_BKV][DH];
  __shared__ float Vs[F32_BKV][DH];
  const AttnWork w = a.work[blockIdx.x];
  const int head = blockIdx.y;
  const int D = a.num_heads * DH;
  const float* base = (const float*)a.qkv;
  const int qrow = w.q0 + threadIdx.x;
  const int seg_end = w.seg_start + w.seg_len;
  const bool qvalid = qrow < seg_end;

  float q[DH], o[DH];
#pragma unroll
  for (int c = 0; c < DH; ++c) {
    q[c] = qvalid ? base[(size_t)qrow * a.ld_qkv + head * DH + c] * a.scale : 0.f;
    o[c] = 0.f;
  }
  float m = -INFINITY, l = 0.f;

  for (int kv0 = w.seg_start; kv0 < seg_end; kv0 += F32_BKV) {
    const int nkv = min(F32_BKV, seg_end - kv0);
    __syncthreads();
    for (int idx = threadIdx.x; idx < F32_BKV * DH; idx += 64) {
      int r = idx / DH, c = idx - r * DH;
      float kvv = 0.f, vv = 0.f;
      if (r < nkv) {
        const float* row = base + (size_t)(kv0 + r) * a.ld_qkv + head * DH + c;
        kvv = row[D];
        vv = row[2 * D];
      }
      Ks[r][c] = kvv;
      Vs[r][c] = vv;
    }
    __syncthreads();
    float sc[F32_BKV];
    float mt = -INFINITY;
#pragma unroll
    for (int j = 0; j < F32_BKV; ++j) {
      float s = 0.f;
#pragma unroll
      for (int c = 0; c < DH; ++c) s = fmaf(q[c], Ks[j][c], s);
      sc[j] = (j < nkv) ? s : -INFINITY;
      mt = fmaxf(mt, sc[j]);
    }
    float mn = fmaxf(m, mt);
    float alpha = expf(m - mn);      // first tile: exp(-inf) = 0
    l *= alpha;
#pragma unroll
    for (int c = 0; c < DH; ++c) o[c] *= alpha;
#pragma unroll
    for (int j = 0; j < F32_BKV; ++j) {
      float p = expf(sc[j] - mn);    // masked entries: exp(-inf) = 0
      l += p;
#pragma unroll
      for (int c = 0; c < DH; ++c) o[c] = fmaf(p, Vs[j][c], o[c]);
    }
    m = mn;
  }
  if (qvalid) {
    float inv = 1.0f / l;
    float* orow = (float*)a.out + (size_t)qrow * a.ld_out + head * DH;
#pragma unroll
    for (int c = 0; c < DH; ++c) orow[c] = o[c] * inv;
  }
}

bool launch_attn_f32(const AttnArgs& a, hipStream_t s) {
  if (a.num_work <= 0) return true;
  dim3 grid(a.num_work, a.num_heads), block(64);
#define EPD_ATTN_F32(DH)                                                   \
  case DH:                                                                 \
    hipLaunchKernelGGL(attn_f32_kernel<DH>, grid, block, 0, s, a);         \
    return true
  switch (a.head_dim) {
    EPD_ATTN_F32(8);
    EPD_ATTN_F32(16);
    EPD_ATTN_F32(32);
    EPD_ATTN_F32(64);
    EPD_ATTN_F32(72);
    EPD_ATTN_F32(80);
    EPD_ATTN_F32(96);
    EPD_ATTN_F32(128);
    default:
      return false;
  }
#undef EPD_ATTN_F32
}

}  // namespace epd
