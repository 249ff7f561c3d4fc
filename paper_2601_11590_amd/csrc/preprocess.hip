// The step in front of the encoder (paper section 3.1: the Encode stage takes the raw
// multimodal input I_m): uint8 pixels -> bilinear resize to the item's patch grid ->
// per-channel normalise -> packed patch rows, the A operand of the patch-embedding GEMM.
//
// The paper does not say how I_m becomes encoder input; this kernel fixes: planar uint8
// frames [C, t*tp, Hs, Ws] per item, bilinear taps at half-pixel centres with the source
// coordinate clamped to the image (no antialiasing, no resampling in time), value
// (v / 255 - mean_c) / std_c, row layout (channel, frame in patch, row in patch, column in
// patch), tokens in raster order over (t, h, w).
//
// Bound: HBM (1 byte in per source pixel, 2 or 4 bytes out per element).  One thread makes
// two neighbouring elements of a patch row (one 4- or 8-byte store); the tap positions are
// exact integer arithmetic, (2j + 1) * n_in - n_out over 2 * n_out, so that equal sizes copy
// pixels untouched and the weights carry a single rounding.
#include "epd_internal.h"

namespace epd {

struct Tap { int i0, i1; float w1; };

// taps of output sample j along an axis of n_in source and n_out output samples
__device__ __forceinline__ Tap tap(int j, int n_in, int n_out) {
  const int num = max((2 * j + 1) * n_in - n_out, 0), den = 2 * n_out;
  Tap t;
  t.i0 = min(num / den, n_in - 1);
  t.i1 = min(t.i0 + 1, n_in - 1);
  t.w1 = (float)(num - (num / den) * den) / (float)den;
  return t;
}

__global__ __launch_bounds__(256) void preprocess_kernel(PrepArgs a) {
  // which item this block works on (at most kPrepItems, ascending block offsets)
  int it = 0;
  while (it + 1 < a.n_items && (int)blockIdx.x >= a.item[it + 1].blk_off) ++it;
  const PrepItem d = a.item[it];
  const long long e = ((long long)(blockIdx.x - d.blk_off) * 256 + threadIdx.x) * 2;   // element pair inside the item
  const long long n_el = (long long)d.t * d.h * d.w * a.pdim;
  if (e >= n_el) return;
  const int p = a.patch;
  const int tok = (int)(e / a.pdim), k = (int)(e - (long long)tok * a.pdim);
  const int px = k % p, py = (k / p) % p, dt = (k / (p * p)) % a.tp, c = k / (p * p * a.tp);
  const int col = tok % d.w, row = (tok / d.w) % d.h, ti = tok / (d.w * d.h);
  const int ho = d.h * p, wo = d.w * p;
  const Tap ty = tap(row * p + py, d.hs, ho);
  const Tap tx0 = tap(col * p + px, d.ws, wo), tx1 = tap(col * p + px + 1, d.ws, wo);
  const uint8_t* f = a.pixels + d.src_off + ((long long)c * (d.t * a.tp) + (ti * a.tp + dt)) * ((long long)d.hs * d.ws);
  const uint8_t* r0 = f + (long long)ty.i0 * d.ws;
  const uint8_t* r1 = f + (long long)ty.i1 * d.ws;
  auto sample = [&](const Tap& tx) {
    const float top = (1.0f - tx.w1) * (float)r0[tx.i0] + tx.w1 * (float)r0[tx.i1];
    const float bot = (1.0f - tx.w1) * (float)r1[tx.i0] + tx.w1 * (float)r1[tx.i1];
    return fmaf((1.0f - ty.w1) * top + ty.w1 * bot, a.a[c], a.b[c]);
  };
  const float v0 = sample(tx0), v1 = sample(tx1);
  const long long o = (long long)d.tok_off * a.pdim + e;
  if (a.out_bf16) {
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    bf16x2 v;
    v[0] = (__bf16)v0; v[1] = (__bf16)v1;
    *(bf16x2*)((uint16_t*)a.out + o) = v;
  } else {
    *(float2*)((float*)a.out + o) = make_float2(v0, v1);
  }
}

void launch_preprocess(const PrepArgs& a, int blocks, hipStream_t s) {
  if (blocks <= 0) return;
  hipLaunchKernelGGL(preprocess_kernel, dim3(blocks), dim3(256), 0, s, a);
}

}  // namespace epd
