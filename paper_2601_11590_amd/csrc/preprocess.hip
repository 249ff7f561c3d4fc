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

// One block = one token (one output row): thread (x, y) makes V neighbouring elements of row y
// of each of the token's channel x frame slabs of patch x patch elements in turn, so every pass
// writes patch * patch consecutive elements and nothing about an element's position has to be
// divided out of a flat index.  V = 8 (one 16-byte bf16 store) when the patch size allows it,
// else 2.  blockIdx.x counts the tokens of the (at most kPrepItems) items of this launch.
template <int V>
__global__ __launch_bounds__(512) void preprocess_kernel(PrepArgs a) {
  // consecutive block ids go to different XCDs (8, each with its own L2): give every XCD a
  // contiguous eighth of the tokens, so that the neighbouring patches that share a 128-byte line
  // of source pixels fetch it through one L2 instead of eight
  const int nb = gridDim.x;
  const int vb = (blockIdx.x & 7) * (nb >> 3) + min((int)(blockIdx.x & 7), nb & 7) + (blockIdx.x >> 3);
  int it = 0;
  while (it + 1 < a.n_items && vb >= a.item[it + 1].blk_off) ++it;
  const PrepItem d = a.item[it];
  const int p = a.patch;
  const int tok = vb - d.blk_off;                         // token inside the item
  const int col = tok % d.w, row = (tok / d.w) % d.h, ti = tok / (d.w * d.h);
  const int px = threadIdx.x * V, py = threadIdx.y;
  const int ho = d.h * p, wo = d.w * p;
  const int y = row * p + py, x = col * p + px;
  const long long plane = (long long)d.hs * d.ws;
  const bool same = d.hs == ho && d.ws == wo;             // no resize: the taps are the pixels themselves
  Tap ty = {y, y, 0.f}, tx[V];
#pragma unroll
  for (int i = 0; i < V; ++i) tx[i] = Tap{x + i, x + i, 0.f};
  if (!same) {
    ty = tap(y, d.hs, ho);
#pragma unroll
    for (int i = 0; i < V; ++i) tx[i] = tap(x + i, d.ws, wo);
  }
  const long long o_row = (long long)(d.tok_off + tok) * a.pdim + py * p + px;
  for (int c = 0; c < a.channels; ++c) {
    const float ac = a.a[c], bc = a.b[c];
    for (int dt = 0; dt < a.tp; ++dt) {
      const uint8_t* f = a.pixels + d.src_off + ((long long)c * (d.t * a.tp) + (ti * a.tp + dt)) * plane;
      const uint8_t* r0 = f + (long long)ty.i0 * d.ws;
      float v[V];
      if (same) {
#pragma unroll
        for (int i = 0; i < V; ++i) v[i] = fmaf((float)r0[x + i], ac, bc);
      } else {
        const uint8_t* r1 = f + (long long)ty.i1 * d.ws;
#pragma unroll
        for (int i = 0; i < V; ++i) {
          const float top = (1.0f - tx[i].w1) * (float)r0[tx[i].i0] + tx[i].w1 * (float)r0[tx[i].i1];
          const float bot = (1.0f - tx[i].w1) * (float)r1[tx[i].i0] + tx[i].w1 * (float)r1[tx[i].i1];
          v[i] = fmaf((1.0f - ty.w1) * top + ty.w1 * bot, ac, bc);
        }
      }
      const long long o = o_row + (long long)(c * a.tp + dt) * p * p;
      if (a.out_bf16) {
        typedef __attribute__((ext_vector_type(V))) __bf16 bf16xV;
        bf16xV w;
#pragma unroll
        for (int i = 0; i < V; ++i) w[i] = (__bf16)v[i];
        *(bf16xV*)((uint16_t*)a.out + o) = w;
      } else {
        typedef __attribute__((ext_vector_type(V))) float f32xV;
        f32xV w;
#pragma unroll
        for (int i = 0; i < V; ++i) w[i] = v[i];
        *(f32xV*)((float*)a.out + o) = w;
      }
    }
  }
}

void launch_preprocess(const PrepArgs& a, int tokens, hipStream_t s) {
  if (tokens <= 0) return;
  // 16-byte stores need the rows (pdim = C * tp * patch^2 elements) and the buffer 16-byte aligned
  const bool wide = a.patch % 8 == 0 && ((size_t)a.out & (a.out_bf16 ? 15 : 31)) == 0;
  if (wide) hipLaunchKernelGGL(preprocess_kernel<8>, dim3(tokens), dim3(a.patch / 8, a.patch), 0, s, a);
  else hipLaunchKernelGGL(preprocess_kernel<2>, dim3(tokens), dim3(a.patch / 2, a.patch), 0, s, a);
}

}  // namespace epd
