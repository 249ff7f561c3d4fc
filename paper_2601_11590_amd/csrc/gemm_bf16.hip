// bf16 GEMM family of the Encode-stage library (ViT forward, paper section 3.1, Eq. 1):
// patch embedding, QKV projection with rotary epilogue, attention output projection, the
// two MLP GEMMs and the merger projection all are  C[M,N] = A[M,K] * W[N,K]^T (+bias)  with
// different epilogues.  Written for gfx950: 64-lane waves, v_mfma_f32_32x32x16_bf16 (fp32
// accumulate), operand tiles staged through LDS with 16-byte accesses.
//
// Tile scheme.  A block of WAVES_M x WAVES_N waves owns a BM x BN output tile; K advances in
// steps of 64.  Both operands are K-contiguous in memory ("NT" form), so one lane's MFMA
// operand (8 consecutive k of one row) is one 16-byte LDS read; LDS rows are padded by 16
// bytes so the 32 rows read by one instruction fall in distinct bank groups.  The next K
// tile is fetched from global memory into registers while the current one is multiplied;
// blocks are sized so two fit on a compute unit and fill each other's barrier and epilogue
// gaps.
//
// Accumulator orientation.  For a 32x32 MFMA result lane l holds column (l % 32) and rows
// 8*(v/4) + 4*(l/32) + (v%4), v = 0..15.  By default the W fragment is fed as the first
// operand, so "rows" are output columns n and the lane's column is a token m: every lane then
// owns runs of 4 consecutive n of one token -- 16-byte fp32 / 8-byte bf16 row-major stores,
// and the two members of a rotary pair (neighbouring n after the create-time reorder) share
// a lane.  For the V third of the QKV projection the operands are swapped, a lane owns 4
// consecutive tokens of one n, and V is stored transposed ([channel][token]) for the
// attention kernel's second GEMM.
#include "epd_internal.h"

namespace epd {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int BK = 64;
constexpr int LDK = BK + 8;   // LDS row stride in elements (144 bytes)

__device__ __forceinline__ uint2 pack_bf16x4(float a, float b, float c, float d) {
  bf16x2 lo, hi;
  lo[0] = (__bf16)a; lo[1] = (__bf16)b; hi[0] = (__bf16)c; hi[1] = (__bf16)d;
  uint2 r;
  r.x = *(uint32_t*)&lo; r.y = *(uint32_t*)&hi;
  return r;
}

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

// Gaussian CDF through the complementary error function, rational-exponential form of the
// Handbook of Mathematical Functions, 7.1.26 (absolute error of erf below 1.5e-7, far below
// the bf16 rounding of the result).
__device__ __forceinline__ float gelu_erf_fast(float x) {
  const float z = fabsf(x) * 0.70710678118654752440f;
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, z, 1.0f));
  float p = fmaf(1.061405429f, t, -1.453152027f);
  p = fmaf(p, t, 1.421413741f);
  p = fmaf(p, t, -0.284496736f);
  p = fmaf(p, t, 0.254829592f);
  p *= t;
  const float e = __builtin_amdgcn_exp2f(-z * z * 1.44269504088896340736f);
  const float half_erfc = 0.5f * p * e;                 // 0.5 * erfc(|x| / sqrt 2)
  const float cdf = x < 0.f ? half_erfc : 1.0f - half_erfc;
  return x * cdf;
}

__device__ __forceinline__ float gelu_tanh_fast(float x) {
  const float u = 0.79788456080286535588f * fmaf(0.044715f * x * x, x, x);
  const float e = __builtin_amdgcn_exp2f(2.0f * 1.44269504088896340736f * u);
  return x * (1.0f - __builtin_amdgcn_rcpf(1.0f + e));   // x * sigmoid(2u)
}

enum OutKind : int { OUT_BF16 = 0, OUT_F32 = 1 };

template <int BM, int BN, int WAVES_M, int WAVES_N, int EPI, int OUT, bool VMODE, bool GATHER>
__device__ __forceinline__ void gemm_tile(const GemmArgs& g, const int m0, const int n0, __bf16* lds) {
  constexpr int NT = 64 * WAVES_M * WAVES_N;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int CPT_A = BM * (BK / 8) / NT, CPT_W = BN * (BK / 8) / NT;
  static_assert(BM * (BK / 8) % NT == 0 && BN * (BK / 8) % NT == 0, "tile / thread mismatch");

  __bf16* As = lds;
  __bf16* Ws = lds + BM * LDK;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  const int l32 = lane & 31, lg = lane >> 5;

  const __bf16* A = (const __bf16*)g.A;
  const __bf16* W = (const __bf16*)g.W;
  const int kcw = GATHER ? g.K / g.gather_n : g.K;

  // per-thread chunk descriptors: chunk c = p * NT + tid -> row c / 8, k chunk c % 8
  const __bf16* a_src[CPT_A];
  bool a_ok[CPT_A];
  int a_m[CPT_A];
#pragma unroll
  for (int p = 0; p < CPT_A; ++p) {
    const int c = p * NT + tid, row = c >> 3, kc = c & 7;
    const int m = m0 + row;
    a_ok[p] = m < g.M;
    a_m[p] = m;
    a_src[p] = A + (size_t)(a_ok[p] ? m : 0) * g.lda + kc * 8;
  }
  const __bf16* w_src[CPT_W];
  bool w_ok[CPT_W];
#pragma unroll
  for (int p = 0; p < CPT_W; ++p) {
    const int c = p * NT + tid, row = c >> 3, kc = c & 7;
    const int n = n0 + row;
    w_ok[p] = n < g.N;
    w_src[p] = W + (size_t)(w_ok[p] ? n : 0) * g.K + kc * 8;
  }

  uint4 a_reg[CPT_A], w_reg[CPT_W];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int p = 0; p < CPT_A; ++p) {
      const int k = k0 + ((p * NT + tid) & 7) * 8;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (a_ok[p] && k < g.K) {
        if constexpr (GATHER) {
          const int piece = k / kcw;
          const int src = g.gather[(size_t)a_m[p] * g.gather_n + piece];
          v = *(const uint4*)(A + (size_t)src * g.lda + (k - piece * kcw));
        } else {
          v = *(const uint4*)(a_src[p] + k0);
        }
      }
      a_reg[p] = v;
    }
#pragma unroll
    for (int p = 0; p < CPT_W; ++p) {
      const int k = k0 + ((p * NT + tid) & 7) * 8;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (w_ok[p] && k < g.K) v = *(const uint4*)(w_src[p] + k0);
      w_reg[p] = v;
    }
  };
  auto stash = [&]() {
#pragma unroll
    for (int p = 0; p < CPT_A; ++p) {
      const int c = p * NT + tid;
      *(uint4*)(As + (c >> 3) * LDK + (c & 7) * 8) = a_reg[p];
    }
#pragma unroll
    for (int p = 0; p < CPT_W; ++p) {
      const int c = p * NT + tid;
      *(uint4*)(Ws + (c >> 3) * LDK + (c & 7) * 8) = w_reg[p];
    }
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const __bf16* a_rd = As + (wm * WM + l32) * LDK + lg * 8;
  const __bf16* w_rd = Ws + (wn * WN + l32) * LDK + lg * 8;

  const int nk = (g.K + BK - 1) / BK;
  fetch(0);
  for (int kt = 0; kt < nk; ++kt) {
    __syncthreads();
    stash();
    __syncthreads();
    if (kt + 1 < nk) fetch((kt + 1) * BK);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 af[TM], wf[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) af[i] = *(const bf16x8*)(a_rd + i * 32 * LDK + ks * 16);
#pragma unroll
      for (int j = 0; j < TN; ++j) wf[j] = *(const bf16x8*)(w_rd + j * 32 * LDK + ks * 16);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          if constexpr (VMODE)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], wf[j], acc[i][j], 0, 0, 0);
          else
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[j], af[i], acc[i][j], 0, 0, 0);
        }
    }
  }

  // ------------------------------------------------------------------ epilogue
  const uint16_t* bias = (const uint16_t*)g.bias;
  if constexpr (VMODE) {
    // lane: column n, runs of 4 consecutive tokens
    uint16_t* vt = (uint16_t*)g.vt;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int n = n0 + wn * WN + j * 32 + l32;
      if (n >= g.N) continue;
      const float b = bias ? bf16_bits_to_float(bias[n]) : 0.f;
      uint16_t* vrow = vt + (size_t)(n - g.qk_cols) * g.vt_stride;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int m = m0 + wm * WM + i * 32 + q * 8 + lg * 4;
          if (m >= g.M) continue;
          const uint2 pk = pack_bf16x4(acc[i][j][4 * q] + b, acc[i][j][4 * q + 1] + b,
                                       acc[i][j][4 * q + 2] + b, acc[i][j][4 * q + 3] + b);
          if (m + 3 < g.M) {
            const int4 vc = *(const int4*)(g.vcol + m);
            if (vc.w - vc.x == 3) {
              *(uint2*)(vrow + vc.x) = pk;
            } else {
              vrow[vc.x] = (uint16_t)(pk.x & 0xffff); vrow[vc.y] = (uint16_t)(pk.x >> 16);
              vrow[vc.z] = (uint16_t)(pk.y & 0xffff); vrow[vc.w] = (uint16_t)(pk.y >> 16);
            }
          } else {
            const uint16_t e[4] = {(uint16_t)(pk.x & 0xffff), (uint16_t)(pk.x >> 16),
                                   (uint16_t)(pk.y & 0xffff), (uint16_t)(pk.y >> 16)};
            for (int t = 0; t < 4 && m + t < g.M; ++t) vrow[g.vcol[m + t]] = e[t];
          }
        }
    }
  } else {
    // lane: token m, runs of 4 consecutive columns n
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int m = m0 + wm * WM + i * 32 + l32;
      if (m >= g.M) continue;
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int n = n0 + wn * WN + j * 32 + q * 8 + lg * 4;
          if (n >= g.N) continue;     // N is a multiple of 4: a run is in or out as a whole
          float v0 = acc[i][j][4 * q], v1 = acc[i][j][4 * q + 1], v2 = acc[i][j][4 * q + 2], v3 = acc[i][j][4 * q + 3];
          if (bias) {
            const uint2 bb = *(const uint2*)(bias + n);
            v0 += bf16_bits_to_float(bb.x & 0xffff); v1 += bf16_bits_to_float(bb.x >> 16);
            v2 += bf16_bits_to_float(bb.y & 0xffff); v3 += bf16_bits_to_float(bb.y >> 16);
          }
          if constexpr (EPI == EPI_QKV) {
            if (g.rot) {
              const int pr = (n % g.head_dim) >> 1;   // even: two pairs = one 16-byte entry
              const float4 cs = *(const float4*)(g.rot + (size_t)m * g.rot_pairs + pr);
              const float r0 = v0 * cs.x - v1 * cs.y, r1 = v0 * cs.y + v1 * cs.x;
              const float r2 = v2 * cs.z - v3 * cs.w, r3 = v2 * cs.w + v3 * cs.z;
              v0 = r0; v1 = r1; v2 = r2; v3 = r3;
            }
          }
          if constexpr (EPI == EPI_GELU) {
            if (g.act == 0) { v0 = gelu_erf_fast(v0); v1 = gelu_erf_fast(v1); v2 = gelu_erf_fast(v2); v3 = gelu_erf_fast(v3); }
            else { v0 = gelu_tanh_fast(v0); v1 = gelu_tanh_fast(v1); v2 = gelu_tanh_fast(v2); v3 = gelu_tanh_fast(v3); }
          }
          if constexpr (EPI == EPI_RESIDUAL) {
            float4* xp = (float4*)(g.resid + (size_t)m * g.ldr + n);
            float4 x = *xp;
            x.x += v0; x.y += v1; x.z += v2; x.w += v3;
            *xp = x;
          } else if constexpr (OUT == OUT_F32) {
            *(float4*)((float*)g.out + (size_t)m * g.ldo + n) = make_float4(v0, v1, v2, v3);
          } else {
            *(uint2*)((uint16_t*)g.out + (size_t)m * g.ldo + n) = pack_bf16x4(v0, v1, v2, v3);
          }
        }
    }
  }
}

// Consecutive hardware block ids go to different XCDs (8 per chip, each with its own L2).
// Remap so that every XCD walks a contiguous range of tiles, N fastest: neighbouring blocks
// of one XCD then share the same A row panel and sweep W.
__device__ __forceinline__ int xcd_remap(int bid, int nblocks) {
  const int q = nblocks >> 3, r = nblocks & 7;
  const int xcd = bid & 7, idx = bid >> 3;
  return xcd * q + min(xcd, r) + idx;
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int EPI, int OUT, bool GATHER>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N, 2) void gemm_bf16_kernel(GemmArgs g) {
  extern __shared__ __attribute__((aligned(16))) char lds_raw[];
  __bf16* lds = (__bf16*)lds_raw;
  const int tiles_n = (g.N + BN - 1) / BN;
  const int tile = xcd_remap(blockIdx.x, gridDim.x);
  const int m0 = (tile / tiles_n) * BM, n0 = (tile % tiles_n) * BN;
  if constexpr (EPI == EPI_QKV) {
    if (n0 >= g.qk_cols) {
      gemm_tile<BM, BN, WAVES_M, WAVES_N, EPI, OUT, true, false>(g, m0, n0, lds);
      return;
    }
  }
  gemm_tile<BM, BN, WAVES_M, WAVES_N, EPI, OUT, false, GATHER>(g, m0, n0, lds);
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int EPI, int OUT, bool GATHER>
static void launch_cfg(const GemmArgs& g, hipStream_t s) {
  const int tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
  const size_t lds = (size_t)(BM + BN) * LDK * sizeof(__bf16);
  auto kern = gemm_bf16_kernel<BM, BN, WAVES_M, WAVES_N, EPI, OUT, GATHER>;
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, dim3(tiles), dim3(64 * WAVES_M * WAVES_N), lds, s, g);
}

template <int EPI, int OUT, bool GATHER>
static void launch_epi(const GemmArgs& g, hipStream_t s) {
  launch_cfg<256, 128, 2, 2, EPI, OUT, GATHER>(g, s);
}

constexpr int kQkvBN = 128;

void launch_gemm_bf16(const GemmArgs& g, hipStream_t s) {
  if (g.M <= 0 || g.N <= 0) return;
  switch (g.epilogue) {
    case EPI_STORE:
      if (g.gather) launch_epi<EPI_STORE, OUT_BF16, true>(g, s);
      else if (g.out_f32) launch_epi<EPI_STORE, OUT_F32, false>(g, s);
      else launch_epi<EPI_STORE, OUT_BF16, false>(g, s);
      break;
    case EPI_GELU:
      launch_epi<EPI_GELU, OUT_BF16, false>(g, s);
      break;
    case EPI_RESIDUAL:
      launch_epi<EPI_RESIDUAL, OUT_F32, false>(g, s);
      break;
    case EPI_QKV:
      if (g.qk_cols % kQkvBN == 0) {
        launch_epi<EPI_QKV, OUT_BF16, false>(g, s);
      } else {
        // a column tile would straddle the K | V boundary: run the two parts separately
        GemmArgs qk = g;
        qk.N = g.qk_cols;
        launch_epi<EPI_QKV, OUT_BF16, false>(qk, s);
        GemmArgs v = g;
        v.W = (const __bf16*)g.W + (size_t)g.qk_cols * g.K;
        v.bias = g.bias ? (const void*)((const __bf16*)g.bias + g.qk_cols) : nullptr;
        v.N = g.N - g.qk_cols;
        v.qk_cols = 0;
        launch_epi<EPI_QKV, OUT_BF16, false>(v, s);
      }
      break;
  }
}

}  // namespace epd
