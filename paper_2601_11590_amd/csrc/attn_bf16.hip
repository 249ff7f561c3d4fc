// Variable-length, block-diagonal, non-causal flash attention on the bf16 matrix cores of
// gfx950 -- the step of the ViT forward (paper section 3.1, Eq. 1) whose cost is quadratic in
// the visual sequence length (paper section 1).  O = softmax(Q K^T / sqrt(d)) V per segment
// and head, never materialising the score matrix.
//
// Layout of the computation (one block = 4 waves = one tile of query rows of one segment and
// head; a wave owns NQ groups of 32 query rows):
//   * Scores are computed transposed, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16: a lane then
//     holds ONE query column (lane % 32) and 16 key rows per 32x32 tile, so the running
//     maximum and the running sum of the softmax are per-lane scalars; one exchange with
//     lane ^ 32 per key tile completes the maximum, the sums are merged once at the end.
//   * The accumulator layout of S^T (key rows 8*(v/4) + 4*(lane/32) + v%4) is, after rounding
//     to bf16, directly the second MFMA operand of O^T = V^T P^T, provided the first operand
//     (V^T) enumerates the keys in the same order.  V is therefore kept transposed
//     ([channel][token], written that way by the QKV GEMM) and a lane reads its 2 x 4 keys
//     with two 8-byte LDS reads.  No data ever moves between lanes for P.
//   * K tiles ([64 keys][d], 16-byte padded rows) and V^T tiles ([d][64 keys], 8-byte padded
//     rows) are staged through LDS once per block and shared by its 4 waves; Q stays in
//     registers as MFMA operands for the whole kernel.
//   * exp is v_exp_f32 (base 2) with 1/sqrt(d) * log2(e) folded into one fused multiply-add.
// Head dimensions that are not multiples of 16 / 32 are zero-padded inside LDS only.
#include "epd_internal.h"

#include <cstdlib>

namespace epd {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int BKV = 64;

union Frag8 {
  bf16x8 v;
  uint4 u;
  uint2 h[2];
  uint32_t w[4];
};

__device__ __forceinline__ uint32_t pack2(float a, float b) {
  bf16x2 t;
  t[0] = (__bf16)a; t[1] = (__bf16)b;
  return *(uint32_t*)&t;
}

template <int DH, int NQ, int MINBLK>
__global__ __launch_bounds__(256, MINBLK) void attn_bf16_kernel(AttnArgs a) {
  constexpr int KS = (DH + 15) / 16;       // k-steps of the score GEMM
  constexpr int DHP = KS * 16;             // K row length in LDS (zero padded)
  constexpr int DB = (DH + 31) / 32;       // 32-row blocks of O^T
  constexpr int KSTR = DHP + 8;            // K row stride (elements): 16-byte pad
  constexpr int VSTR = BKV + 4;            // V^T row stride (elements): 8-byte pad
  constexpr int BQ = 128 * NQ;

  __shared__ __attribute__((aligned(16))) __bf16 Ks[BKV * KSTR];
  __shared__ __attribute__((aligned(16))) __bf16 Vs[DB * 32 * VSTR];

  const AttnWork w = a.work[blockIdx.x];
  const int head = blockIdx.y;
  const int D = a.num_heads * DH;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lg = lane >> 5;
  const int seg_end = w.seg_start + w.seg_len;
  const uint16_t* qk = (const uint16_t*)a.qkv;
  const uint16_t* vt = (const uint16_t*)a.vt + (size_t)head * DH * a.vt_stride + w.vcol0;

  // zero the LDS padding once (K columns DH..DHP, V^T rows DH..DB*32); loads never touch it
  if constexpr (DHP > DH) {
    for (int i = tid; i < BKV * (DHP - DH); i += 256) {
      const int r = i / (DHP - DH), c = DH + i % (DHP - DH);
      ((uint16_t*)Ks)[r * KSTR + c] = 0;
    }
  }
  if constexpr (DB * 32 > DH) {
    for (int i = tid; i < (DB * 32 - DH) * VSTR; i += 256) ((uint16_t*)Vs)[DH * VSTR + i] = 0;
  }

  // Q fragments (second MFMA operand of S^T = K Q^T): lane = query column, 8 consecutive d
  Frag8 qf[NQ][KS];
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    const int qrow = w.q0 + wave * 32 * NQ + nq * 32 + l32;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int d = ks * 16 + lg * 8;
      qf[nq][ks].u = make_uint4(0, 0, 0, 0);
      if (qrow < seg_end && d < DH) qf[nq][ks].u = *(const uint4*)(qk + (size_t)qrow * a.ld_qkv + head * DH + d);
    }
  }

  f32x16 o[DB][NQ];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
      for (int v = 0; v < 16; ++v) o[db][nq][v] = 0.f;
  float mrun[NQ], lrun[NQ];
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) { mrun[nq] = -INFINITY; lrun[nq] = 0.f; }

  const float c = a.scale * 1.44269504088896340736f;   // scores are handled in log2 units

  for (int kv0 = 0; kv0 < w.seg_len; kv0 += BKV) {
    const int nvalid = w.seg_len - kv0;   // >= 1
    __syncthreads();
    // K tile: 64 rows x DH/8 chunks of 16 bytes
    for (int i = tid; i < BKV * (DH / 8); i += 256) {
      const int r = i / (DH / 8), ch = i % (DH / 8);
      uint4 v = make_uint4(0, 0, 0, 0);
      if (r < nvalid) v = *(const uint4*)(qk + (size_t)(w.seg_start + kv0 + r) * a.ld_qkv + D + head * DH + ch * 8);
      *(uint4*)((uint16_t*)Ks + r * KSTR + ch * 8) = v;
    }
    // V^T tile: DH rows x 8 chunks of 16 bytes (columns beyond the segment are zero in memory)
    for (int i = tid; i < DH * (BKV / 8); i += 256) {
      const int r = i >> 3, ch = i & 7;
      const uint4 v = *(const uint4*)(vt + (size_t)r * a.vt_stride + kv0 + ch * 8);
      uint2* dst = (uint2*)((uint16_t*)Vs + r * VSTR + ch * 8);
      dst[0] = make_uint2(v.x, v.y);
      dst[1] = make_uint2(v.z, v.w);
    }
    __syncthreads();

    // ---- S^T = K Q^T
    f32x16 s[2][NQ];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
        for (int v = 0; v < 16; ++v) s[kb][nq][v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      bf16x8 kf[2];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) kf[kb] = *(const bf16x8*)(Ks + (kb * 32 + l32) * KSTR + ks * 16 + lg * 8);
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq)
          s[kb][nq] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kb], qf[nq][ks].v, s[kb][nq], 0, 0, 0);
    }
    if (nvalid < BKV) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int kvl = kb * 32 + 8 * (v >> 2) + 4 * lg + (v & 3);
          if (kvl >= nvalid) {
#pragma unroll
            for (int nq = 0; nq < NQ; ++nq) s[kb][nq][v] = -INFINITY;
          }
        }
    }

    // ---- online softmax, per query column (= per lane pair l, l ^ 32)
    Frag8 pb[NQ][2][2];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
      float mx = s[0][nq][0];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[kb][nq][v]);
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float mnew = fmaxf(mrun[nq], mx * c);
      const float alpha = __builtin_amdgcn_exp2f(mrun[nq] - mnew);
      mrun[nq] = mnew;
      float psum = 0.f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int mm = 0; mm < 2; ++mm)
#pragma unroll
          for (int e = 0; e < 8; e += 2) {
            const float p0 = __builtin_amdgcn_exp2f(fmaf(s[kb][nq][8 * mm + e], c, -mnew));
            const float p1 = __builtin_amdgcn_exp2f(fmaf(s[kb][nq][8 * mm + e + 1], c, -mnew));
            psum += p0 + p1;
            pb[nq][kb][mm].w[e >> 1] = pack2(p0, p1);
          }
      lrun[nq] = lrun[nq] * alpha + psum;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[db][nq][v] *= alpha;
    }

    // ---- O^T += V^T P^T
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int mm = 0; mm < 2; ++mm) {
          Frag8 vf;
          const uint16_t* src = (const uint16_t*)Vs + (db * 32 + l32) * VSTR + kb * 32 + 16 * mm + 4 * lg;
          vf.h[0] = *(const uint2*)src;
          vf.h[1] = *(const uint2*)(src + 8);
#pragma unroll
          for (int nq = 0; nq < NQ; ++nq)
            o[db][nq] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.v, pb[nq][kb][mm].v, o[db][nq], 0, 0, 0);
        }
  }

  // ---- normalise and store: lane owns runs of 4 consecutive channels of one query row
  uint16_t* out = (uint16_t*)a.out;
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    const int qrow = w.q0 + wave * 32 * NQ + nq * 32 + l32;
    const float ltot = lrun[nq] + __shfl_xor(lrun[nq], 32);
    if (qrow >= seg_end) continue;
    const float inv = 1.0f / ltot;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int d = db * 32 + q * 8 + lg * 4;
        if (d >= DH) continue;
        uint2 pk;
        pk.x = pack2(o[db][nq][4 * q] * inv, o[db][nq][4 * q + 1] * inv);
        pk.y = pack2(o[db][nq][4 * q + 2] * inv, o[db][nq][4 * q + 3] * inv);
        *(uint2*)(out + (size_t)qrow * a.ld_out + head * DH + d) = pk;
      }
  }
}

static int bf16_nq() {
  static int nq = [] {
    const char* e = getenv("EPD_ATTN_NQ");
    return (e && e[0] == '1') ? 1 : 2;
  }();
  return nq;
}

int attn_q_tile(bool bf16, int head_dim) {
  if (!bf16) {
    switch (head_dim) {
      case 8: case 16: case 32: case 64: case 72: case 80: case 96: case 128: return 64;
      default: return 0;
    }
  }
  switch (head_dim) {
    case 32: case 64: case 72: case 80: case 96: case 128: return 128 * bf16_nq();
    default: return 0;
  }
}

bool launch_attn_bf16(const AttnArgs& a, hipStream_t s) {
  if (a.num_work <= 0) return true;
  dim3 grid(a.num_work, a.num_heads), block(256);
  const int nq = bf16_nq();
#define EPD_ATTN(DH, MB2)                                                                    \
  case DH:                                                                                   \
    if (nq == 2) hipLaunchKernelGGL((attn_bf16_kernel<DH, 2, MB2>), grid, block, 0, s, a);   \
    else hipLaunchKernelGGL((attn_bf16_kernel<DH, 1, 2>), grid, block, 0, s, a);             \
    return true
  switch (a.head_dim) {
    EPD_ATTN(32, 2);
    EPD_ATTN(64, 2);
    EPD_ATTN(72, 1);
    EPD_ATTN(80, 1);
    EPD_ATTN(96, 1);
    EPD_ATTN(128, 1);
    default:
      return false;
  }
#undef EPD_ATTN
}

}  // namespace epd
