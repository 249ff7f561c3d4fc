// Variable-length, block-diagonal, non-causal flash attention on the bf16 matrix cores of
// gfx950 -- the step of the ViT forward (paper section 3.1, Eq. 1) whose cost is quadratic in
// the visual sequence length (paper section 1).  O = softmax(Q K^T / sqrt(d)) V per segment
// and head, never materialising the score matrix.
//
// Layout of the computation (one block = NW waves (4 or 8) = one tile of query rows of one
// segment and head; a wave owns NQ groups of 32 query rows):
//   * Scores are computed transposed, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16: a lane then
//     holds ONE query column (lane % 32) and 16 key rows per 32x32 tile, so the running
//     maximum and the running sum of the softmax are per-lane scalars; one exchange between
//     the two lane halves (v_permlane32_swap) per key tile completes the maximum, the sums
//     are merged once at the end.
//   * The accumulator layout of S^T (rows 8*(v/4) + 4*(lane/32) + v%4) is, after rounding to
//     bf16, directly the second MFMA operand of O^T = V^T P^T, provided the first operand
//     (V^T) enumerates the keys in the same order.  A lane's accumulator rows come in runs of
//     four, eight apart; the K tile is therefore laid out in LDS with rows 4-7 and 8-11 of
//     every 16 exchanged (row r holds key r with bits 2 and 3 swapped -- free, since every
//     lane of a direct-to-LDS load picks its own source row), which makes the eight values a
//     lane feeds into one MFMA eight CONSECUTIVE keys.  V is kept transposed ([channel][token],
//     written that way by the QKV GEMM) in natural key order, and a lane reads its 8 keys with
//     one 16-byte LDS read.  No data ever moves between lanes for P.
//   * K tiles ([64 keys][d]) and V^T tiles ([d][64 keys]) go from global memory straight into
//     LDS (global_load_lds_dwordx4) in a two-stage ring: the tile after the current one is in
//     flight while the current one is multiplied, one barrier per key tile.  Rows of 128 bytes
//     are XOR-swizzled at 16-byte granularity for the 64-bank LDS; fragment reads are
//     explicit ds_read instructions with counted waits so that they are never serialised
//     against the loads in flight.  Q stays in registers as MFMA operands for the whole kernel.
//   * exp is v_exp_f32 (base 2) with 1/sqrt(d) * log2(e) folded into one fused multiply-add;
//     the softmax reference value trails the running maximum by up to 8 (log2 units), so the
//     output accumulators are rescaled only rarely (and then for the whole wave).
// Head dimensions that are not multiples of 16 / 32 are handled by zeroing the Q operand
// beyond d and never storing output rows beyond d; where the channels beyond the last whole
// 32-row block of O^T fit 16 rows (d = 72) that block is computed with
// v_mfma_f32_16x16x32_bf16, whose second operand is made from the probability registers by
// exchanging 16-lane rows (v_permlane16_swap).
#include "epd_internal.h"

#include <type_traits>

namespace epd {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

#define EPD_GPTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define EPD_LPTR(p) ((__attribute__((address_space(3))) void*)(p))

constexpr int BKV = 64;
constexpr float kLag = 8.0f;   // slack of the running softmax reference, in log2 units

union Frag8 {
  bf16x8 v;
  uint4 u;
  uint32_t w[4];
};

__device__ __forceinline__ uint32_t pack2(float a, float b) {
  bf16x2 t;
  t[0] = (__bf16)a; t[1] = (__bf16)b;
  return *(uint32_t*)&t;
}

template <int OFF> __device__ __forceinline__ void lds_read16(bf16x8& d, uint32_t addr) {
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(d) : "v"(addr), "n"(OFF) : "memory");
}
// The compiler takes the result of an inline ds_read for valid at once; the ties that follow a
// wait keep the consumers behind it, and the scheduling barrier keeps any register copy the
// compiler makes for a tie behind it as well (a copy hoisted above the wait would read a
// register the LDS has not filled yet).  The generated code is checked for such copies at
// build time (check_lds_waits.py).
template <int PENDING> __device__ __forceinline__ void lds_wait() {
  asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(PENDING) : "memory");
  __builtin_amdgcn_sched_barrier(0);
}
__device__ __forceinline__ void tie(bf16x8& f) { asm volatile("" : "+v"(f)); }

// Key (within its tile) held by row r of the K tile in LDS: bits 2 and 3 of r exchanged.
__device__ __forceinline__ constexpr int key_of_row(int r) { return (r & ~12) | ((r & 4) << 1) | ((r & 8) >> 1); }

// max over the two halves of the wave (lane l and lane l ^ 32)
__device__ __forceinline__ float half_swap_max(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_swap_sum(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

template <int DH, int NQ, int MINBLK, bool SUMROW, int NW>
__global__ __launch_bounds__(64 * NW, MINBLK) void attn_bf16_kernel(AttnArgs a) {
  constexpr int NT = 64 * NW;              // threads per block
  constexpr int KS = (DH + 15) / 16;       // k-steps of the score GEMM
  constexpr int DB = (DH + 31) / 32;       // 32-row blocks of O^T that hold output channels
  // SUMROW: row DH of the V^T tile in LDS is a row of ones, so that row DH of O^T accumulates
  // the softmax denominator in the matrix cores (rescaled together with the outputs) instead
  // of 32 vector additions per key tile
  constexpr int DBX = SUMROW ? (DH + 32) / 32 : DB;   // 32-row blocks of O^T that hold channels or the ones row
  // TAIL16: the channels beyond the last whole 32-row block, and the ones row, fit 16 rows
  // (d = 72: channels 64 .. 71 and the ones row).  That block of O^T is then computed with
  // v_mfma_f32_16x16x32_bf16 -- two 16-query blocks x 32 keys -- at half the matrix-core time
  // of a 32-row block that would be three quarters padding.
  constexpr bool TAIL16 = SUMROW && NQ == 1 && (DH % 32) != 0 && (DH % 32) + 1 <= 16;
  constexpr int DBF = TAIL16 ? DH / 32 : DBX;         // 32-row blocks of O^T computed with the 32x32x16 form
  constexpr int VROWS = TAIL16 ? DBF * 32 + 16 : DBX * 32;
  constexpr int CPRK = DH / 8;             // 16-byte chunks per K row
  constexpr int ROWK = DH * 2;             // bytes per K row in LDS
  constexpr int KBYTES = BKV * ROWK;
  constexpr int VBYTES = VROWS * 128;      // V^T tile: DH rows of 64 keys, padded to whole blocks of rows
  constexpr int STAGE = KBYTES + VBYTES;
  constexpr int LK = (BKV * CPRK + NT - 1) / NT, LV = (DH * 8 + NT - 1) / NT;
  // K row swizzle: power-of-two rows need one (all rows would start in the same banks);
  // 144-byte rows (d = 72) already spread 16 consecutive rows over all 64 banks
  constexpr bool SWZK = (CPRK & (CPRK - 1)) == 0;
  // slack: the K fragment read of a padded head dim runs one chunk past the tile; what it
  // fetches only meets zero Q operands
  __shared__ __attribute__((aligned(1024))) char lds[2 * STAGE + 64];

  // blocks are dealt round-robin to the 8 XCDs, each with its own L2: XCD x takes the x-th
  // contiguous eighth of the (head, work item) list, so that the query tiles of one segment
  // and head -- which read the same K and V^T -- run side by side behind one L2
  const int nblk = gridDim.x;
  const int vb = (blockIdx.x & 7) * (nblk >> 3) + min((int)(blockIdx.x & 7), nblk & 7) + (blockIdx.x >> 3);
  const int head = vb / a.num_work;
  const AttnWork w = a.work[vb - head * a.num_work];
  const int D = a.num_heads * DH;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, lg = lane >> 5;
  const int seg_end = w.seg_start + w.seg_len;
  const uint16_t* qk = (const uint16_t*)a.qkv;
  const char* kbase = (const char*)(qk + (size_t)w.seg_start * a.ld_qkv + D + head * DH);
  const char* vbase = (const char*)((const uint16_t*)a.vt + (size_t)head * DH * a.vt_stride + w.vcol0);
  const int ntiles = (w.seg_len + BKV - 1) / BKV;

  // V^T rows DH .. VROWS-1 of both stages are never loaded: row DH becomes the row of ones
  // (SUMROW), the others zero, once, before the first barrier
  if constexpr (VROWS > DH) {
    constexpr int PADCH = (VROWS - DH) * 8;      // 16-byte chunks per stage
    for (int i = threadIdx.x; i < 2 * PADCH; i += NT) {
      const int st = i / PADCH, ch = i - st * PADCH;
      const uint32_t fill = (SUMROW && ch < 8) ? 0x3F803F80u : 0u;   // bf16 1.0 pairs
      *(uint4*)(lds + st * STAGE + KBYTES + DH * 128 + ch * 16) = make_uint4(fill, fill, fill, fill);
    }
  }

  // ---- load descriptors (direct-to-LDS: lane i of an instruction fills LDS chunk base + i)
  int k_row[LK], k_ch[LK];
  bool k_on[LK];
#pragma unroll
  for (int it = 0; it < LK; ++it) {
    const int lin = it * NT + tid;
    k_on[it] = lin < BKV * CPRK;
    const int row = lin / CPRK, slot = lin - row * CPRK;
    k_row[it] = key_of_row(row);   // LDS row `row` receives this key of the tile
    k_ch[it] = SWZK ? (slot ^ ((CPRK == 8 ? (row >> 1) : row) & (CPRK - 1))) : slot;
  }
  uint32_t v_off[LV];
  bool v_on[LV];
#pragma unroll
  for (int it = 0; it < LV; ++it) {
    const int lin = it * NT + tid;
    v_on[it] = lin < DH * 8;
    const int row = lin >> 3, slot = lin & 7;
    v_off[it] = (uint32_t)row * (uint32_t)a.vt_stride * 2u + (uint32_t)((slot ^ ((row >> 1) & 7)) * 16);
  }
  auto issue = [&](int st, int tile) {
    char* sb = lds + st * STAGE;
    const int kv0 = tile * BKV;
#pragma unroll
    for (int it = 0; it < LK; ++it) {
      if (k_on[it]) {
        const int r = min(kv0 + k_row[it], w.seg_len - 1);   // rows past the segment repeat its last key (masked later)
        // scalar base + 32-bit lane offset: the load's own addressing form, no 64-bit vector
        // arithmetic (a segment's K rows span far less than 4 GB)
        const uint32_t off = (uint32_t)r * (uint32_t)(a.ld_qkv * 2) + (uint32_t)(k_ch[it] * 16);
        __builtin_amdgcn_global_load_lds(EPD_GPTR(kbase + (size_t)off), EPD_LPTR(sb + (it * NT + wave * 64) * 16), 16, 0, 0);
      }
    }
    const char* vb = vbase + (size_t)kv0 * 2;
#pragma unroll
    for (int it = 0; it < LV; ++it) {
      if (v_on[it]) {
        uint32_t off = v_off[it];
        asm volatile("" : "+v"(off));        // keeps the widening to 64 bits next to the load (same form as above)
        __builtin_amdgcn_global_load_lds(EPD_GPTR(vb + (size_t)off), EPD_LPTR(sb + KBYTES + (it * NT + wave * 64) * 16), 16, 0, 0);
      }
    }
  };

  // ---- fragment read addresses (stage 0; stage 1 and row blocks through the offset field)
  const uint32_t lds0 = (uint32_t)(size_t)EPD_LPTR(lds);
  uint32_t k_rd[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    const int ch = ks * 2 + lg;
    const int slot = SWZK ? (ch ^ ((CPRK == 8 ? (l32 >> 1) : l32) & (CPRK - 1))) : ch;
    k_rd[ks] = lds0 + l32 * ROWK + slot * 16;
  }
  // V^T fragment f = kb*2 + mm: keys 16 f + 8 lg .. + 7 of channel row l32 = 16-byte chunk
  // 2 f + lg of that row (row blocks of 32 keep the swizzle)
  uint32_t v_rd[4];
#pragma unroll
  for (int f = 0; f < 4; ++f) v_rd[f] = lds0 + KBYTES + l32 * 128 + (((2 * f + lg) ^ ((l32 >> 1) & 7)) * 16);
  // TAIL16: first operand of the 16x16x32 form = 16 rows x 32 keys, lane (l16, g4) supplies 8 keys
  // of row l16.  The second operand is made from the two 16-key probability fragments of a
  // 32-key block by exchanging 16-lane rows (see compute), which puts keys 0-7 | 16-23 | 8-15 |
  // 24-31 of the block into lane groups g4 = 0 | 1 | 2 | 3: the V^T fragment follows that order,
  // 16-byte chunk 4 kb + {0, 2, 1, 3}[g4] of row DBF*32 + l16 (kb = 1: address bit 6 flipped).
  const int l16 = lane & 15, g4 = lane >> 4;
  [[maybe_unused]] const uint32_t vt_rd = lds0 + KBYTES + (DBF * 32 + l16) * 128 +
                                          (((((g4 & 1) << 1) | (g4 >> 1)) ^ (((DBF * 32 + l16) >> 1) & 7)) * 16);

  // a wave none of whose query rows exist still takes part in loads and barriers only
  const int q_wave0 = w.q0 + wave * 32 * NQ;
  const bool wave_active = q_wave0 < seg_end;

  // Q fragments (second MFMA operand of S^T = K Q^T): lane = query column, 8 consecutive d
  Frag8 qf[NQ][KS];
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    const int qrow = q_wave0 + nq * 32 + l32;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int d = ks * 16 + lg * 8;
      qf[nq][ks].u = make_uint4(0, 0, 0, 0);
      if (qrow < seg_end && d < DH) qf[nq][ks].u = *(const uint4*)(qk + (size_t)qrow * a.ld_qkv + head * DH + d);
    }
  }

  f32x16 o[DBF][NQ];
#pragma unroll
  for (int db = 0; db < DBF; ++db)
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
      for (int v = 0; v < 16; ++v) o[db][nq][v] = 0.f;
  // TAIL16: ot[b] = rows DBF*32 .. +15 of O^T for queries 16 b + l16; lane (l16, g4) holds rows
  // 4 g4 .. 4 g4 + 3 (channels in g4 = 0, 1; the ones row = softmax denominator in g4 = 2, v = 0)
  [[maybe_unused]] f32x4 ot[2];
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int v = 0; v < 4; ++v) ot[b][v] = 0.f;
  float mrun[NQ], lrun[NQ];
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) { mrun[nq] = -INFINITY; lrun[nq] = 0.f; }

  // Q arrives multiplied by 1/sqrt(d) * log2(e) (folded into the QKV projection before its
  // bf16 rounding), so K Q^T already is the score in log2 units.
  // CREF (one 32-row group per wave): the softmax reference is subtracted inside the matrix
  // cores -- the first MFMA of a score tile starts from an accumulator preset to -reference --
  // so that a probability is exp2 of the accumulator itself, without a multiply-add per score.
  // The preset only changes when the reference moves (rare, see kLag).  It costs 16 registers
  // per 32-row group: used where that does not lower the occupancy (d >= 72: +3-6 % measured;
  // at d = 64 the kernel would drop from three to two waves per SIMD and lose 5 %).
  constexpr bool CREF = NQ == 1 && DH >= 72;
  f32x16 cref[NQ];
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
    for (int v = 0; v < 16; ++v) cref[nq][v] = 0.f;

  auto compute = [&](auto ST, int nvalid, const bool first) {
    constexpr int st = decltype(ST)::value;
    constexpr int SO = st * STAGE;
    // ---- S^T = K Q^T: K fragments of k-step ks+1 are requested before step ks is multiplied
    f32x16 s[2][NQ];
    if constexpr (!CREF) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
          for (int v = 0; v < 16; ++v) s[kb][nq][v] = 0.f;
    }
    bf16x8 kf[2][2];
    lds_read16<SO>(kf[0][0], k_rd[0]);
    lds_read16<SO + 32 * ROWK>(kf[0][1], k_rd[0]);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int cur = ks & 1;
      if (ks + 1 < KS) {
        lds_read16<SO>(kf[cur ^ 1][0], k_rd[ks + 1 < KS ? ks + 1 : 0]);
        lds_read16<SO + 32 * ROWK>(kf[cur ^ 1][1], k_rd[ks + 1 < KS ? ks + 1 : 0]);
        lds_wait<2>();
      } else {
        lds_wait<0>();
      }
      tie(kf[cur][0]); tie(kf[cur][1]);
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq) {
          if (CREF && ks == 0) s[kb][nq] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[cur][kb], qf[nq][ks].v, cref[nq], 0, 0, 0);
          else s[kb][nq] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[cur][kb], qf[nq][ks].v, s[kb][nq], 0, 0, 0);
        }
    }
    if (nvalid < BKV) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int kvl = kb * 32 + key_of_row(8 * (v >> 2) + (v & 3)) + 8 * lg;   // key of accumulator row 8 (v/4) + 4 lg + v%4
          if (kvl >= nvalid) {
#pragma unroll
            for (int nq = 0; nq < NQ; ++nq) s[kb][nq][v] = -INFINITY;
          }
        }
    }

    // ---- online softmax, per query column (= per lane pair l, l ^ 32)
    // The reference only follows the true maximum when it falls behind by more than kLag (log2
    // units): in between, probabilities may reach 2^kLag instead of 1, which fp32 sums and bf16
    // operands hold without loss, and nothing needs rescaling.
    Frag8 pb[NQ][2][2];
    float alpha[NQ], delta[NQ];
    bool moved = false;
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
      float mx = s[0][nq][0];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[kb][nq][v]);
      mx = half_swap_max(mx);
      if constexpr (CREF) {
        // mx = true maximum - reference (the very first tile is measured against reference 0)
        const bool lag = first || mx > kLag;
        delta[nq] = lag ? mx : 0.f;
        alpha[nq] = first ? 0.f : __builtin_amdgcn_exp2f(-delta[nq]);
        moved = moved || lag;
        mrun[nq] = (first ? 0.f : mrun[nq]) + delta[nq];
      } else {
        const bool lag = mx > mrun[nq] + kLag;
        const float mnew = lag ? mx : mrun[nq];
        alpha[nq] = __builtin_amdgcn_exp2f(mrun[nq] - mnew);
        moved = moved || lag;
        mrun[nq] = mnew;
        delta[nq] = mnew;      // subtracted from every score below
      }
    }
    const bool any_moved = __builtin_amdgcn_ballot_w64(moved) != 0;
    auto probs = [&](auto SUBT) {
      constexpr bool sub = decltype(SUBT)::value;
#pragma unroll
      for (int nq = 0; nq < NQ; ++nq) {
        float psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int mm = 0; mm < 2; ++mm)
#pragma unroll
            for (int e = 0; e < 8; e += 2) {
              const float x0 = s[kb][nq][8 * mm + e], x1 = s[kb][nq][8 * mm + e + 1];
              const float p0 = __builtin_amdgcn_exp2f(sub ? x0 - delta[nq] : x0);
              const float p1 = __builtin_amdgcn_exp2f(sub ? x1 - delta[nq] : x1);
              if constexpr (!SUMROW) psum += p0 + p1;
              pb[nq][kb][mm].w[e >> 1] = pack2(p0, p1);
            }
        if constexpr (!SUMROW) lrun[nq] = lrun[nq] * alpha[nq] + psum;
      }
    };
    if (!CREF || any_moved) probs(std::true_type{}); else probs(std::false_type{});
    // rescale the output accumulators (and renew the accumulator preset) only if some row's
    // reference moved (wave-uniform test)
    if (any_moved) {
#pragma unroll
      for (int nq = 0; nq < NQ; ++nq) {
#pragma unroll
        for (int db = 0; db < DBF; ++db)
#pragma unroll
          for (int v = 0; v < 16; ++v) o[db][nq][v] *= alpha[nq];
        if constexpr (TAIL16) {
          // a lane holds the factor of query lane % 32; the 16-query blocks need those of queries
          // l16 and 16 + l16 in all four lane groups: one exchange of 16-lane rows yields both
          const auto ab = __builtin_amdgcn_permlane16_swap(__float_as_uint(alpha[nq]), __float_as_uint(alpha[nq]), false, false);
#pragma unroll
          for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 4; ++v) ot[b][v] *= __uint_as_float(ab[b]);
        }
        if constexpr (CREF) {
#pragma unroll
          for (int v = 0; v < 16; ++v) cref[nq][v] = -mrun[nq];
        }
      }
    }

    // ---- O^T += V^T P^T: fragments of one 32-channel block are requested ahead of its MFMAs
    Frag8 vf[2][4];
    auto read_v = [&](auto DBI, int buf) {
      constexpr int off = SO + decltype(DBI)::value * 32 * 128;
#pragma unroll
      for (int f = 0; f < 4; ++f) lds_read16<off>(vf[buf][f].v, v_rd[f]);   // f = kb*2 + mm
    };
    auto pv = [&](int db, int buf) {
#pragma unroll
      for (int f = 0; f < 4; ++f) {
        tie(vf[buf][f].v);
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq)
          o[db][nq] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[buf][f].v, pb[nq][f >> 1][f & 1].v, o[db][nq], 0, 0, 0);
      }
    };
    [[maybe_unused]] bf16x8 vt[2];
    auto pv_blocks = [&](auto self, auto DBI) {
      constexpr int db = decltype(DBI)::value;
      if constexpr (db < DBF) {
        if constexpr (db + 1 < DBF) {
          read_v(std::integral_constant<int, db + 1>{}, (db + 1) & 1);
          lds_wait<4>();
        } else if constexpr (TAIL16) {
          lds_read16<SO>(vt[0], vt_rd);
          lds_read16<SO>(vt[1], vt_rd ^ 64u);
          lds_wait<2>();
        } else {
          lds_wait<0>();
        }
        pv(db, db & 1);
        self(self, std::integral_constant<int, db + 1>{});
      }
    };
    read_v(std::integral_constant<int, 0>{}, 0);
    pv_blocks(pv_blocks, std::integral_constant<int, 0>{});
    if constexpr (TAIL16) {
      lds_wait<0>();
      tie(vt[0]); tie(vt[1]);
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        // x: keys 8 lg .. + 7, y: keys 16 + 8 lg .. + 7 of the block, for query lane % 32.  The
        // exchange gives x the rows (x0, y0, x2, y2) -- queries 0 .. 15 in every lane group, keys
        // 0-7 | 16-23 | 8-15 | 24-31 -- and y the rows (x1, y1, x3, y3): queries 16 .. 31.
        Frag8 x = pb[0][kb][0], y = pb[0][kb][1];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const auto r = __builtin_amdgcn_permlane16_swap(x.w[i], y.w[i], false, false);
          x.w[i] = r[0]; y.w[i] = r[1];
        }
        ot[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vt[kb], x.v, ot[0], 0, 0, 0);
        ot[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vt[kb], y.v, ot[1], 0, 0, 0);
      }
    }
  };

  // ---- key tiles: two-stage ring, the next tile is in flight while this one is multiplied
  issue(0, 0);
  for (int j = 0; j < ntiles; j += 2) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    if (j + 1 < ntiles) issue(1, j + 1);
    if (wave_active) compute(std::integral_constant<int, 0>{}, w.seg_len - j * BKV, j == 0);
    if (j + 1 < ntiles) {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __builtin_amdgcn_s_barrier();
      if (j + 2 < ntiles) issue(0, j + 2);
      if (wave_active) compute(std::integral_constant<int, 1>{}, w.seg_len - (j + 1) * BKV, false);
    }
  }

  // ---- normalise and store: lane owns runs of 4 consecutive channels of one query row
  uint16_t* out = (uint16_t*)a.out;
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    const int qrow = q_wave0 + nq * 32 + l32;
    float ltot;
    if constexpr (TAIL16) {
      // the denominators of queries l16 / 16 + l16 stand in lanes 32 + l16 of ot[0] / ot[1]
      // (row 8 of the block = the ones row): bring them to lane groups 0 and 2, then to all four
      const float t0 = ot[0][0], t1 = ot[1][0];
      const auto h0 = __builtin_amdgcn_permlane32_swap(__float_as_uint(t0), __float_as_uint(t0), false, false);
      const auto h1 = __builtin_amdgcn_permlane32_swap(__float_as_uint(t1), __float_as_uint(t1), false, false);
      const float w0 = __uint_as_float(__builtin_amdgcn_permlane16_swap(h0[1], h0[1], false, false)[0]);
      const float w1 = __uint_as_float(__builtin_amdgcn_permlane16_swap(h1[1], h1[1], false, false)[0]);
      ltot = l32 < 16 ? w0 : w1;
      // channels DBF*32 + 4 g4 .. + 3 of queries 16 b + l16 (lane groups that hold channels)
      if (4 * g4 < DH - DBF * 32) {
#pragma unroll
        for (int b = 0; b < 2; ++b) {
          const int qr = q_wave0 + 16 * b + l16;
          if (qr >= seg_end) continue;
          const float inv = 1.0f / (b ? w1 : w0);
          uint2 pk;
          pk.x = pack2(ot[b][0] * inv, ot[b][1] * inv);
          pk.y = pack2(ot[b][2] * inv, ot[b][3] * inv);
          *(uint2*)(out + (size_t)qr * a.ld_out + head * DH + DBF * 32 + 4 * g4) = pk;
        }
      }
    } else if constexpr (SUMROW) {
      // row DH of O^T: block DH / 32, row r = DH % 32 -> accumulator register 4*(r/8) + r%4 of
      // the lanes of half (r % 8) / 4; the swap hands both halves' values to every lane
      constexpr int r = DH % 32;
      const float x = o[DH / 32][nq][4 * (r / 8) + (r % 4)];
      const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
      ltot = __uint_as_float(sw[(r % 8) / 4]);
    } else {
      ltot = half_swap_sum(lrun[nq]);
    }
    if (qrow >= seg_end) continue;
    const float inv = 1.0f / ltot;
#pragma unroll
    for (int db = 0; db < (TAIL16 ? DBF : DB); ++db)
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

// Query rows per work item: 128 (four waves of one 32-row group) or 256.  For d <= 64 the 256-row
// tile is four waves of TWO groups each, which halves the LDS fragment traffic per MFMA and wins
// on long segments; the one-group kernels for d <= 64 are compiled for four waves per SIMD (128
// registers, which the compiler meets with one spilled register): +6-10 % over three, and a batch
// of eight 784-token images x 16 heads (3200 wave tasks) then fits the chip's 4096 wave slots in
// one round.  Larger head dims have no registers for two groups per wave at two waves per SIMD;
// their 256-row tile is EIGHT waves of one group -- one block per compute unit instead of two, so
// every K / V^T tile is loaded once for 256 query rows: +4 % at d = 72 on a 28 224-token segment,
// nothing at d = 128 (where it is kept for tuning and tests only).  Short segments keep the
// 128-row tile, which wastes less on their tails.
static int bf16_q_rows(int head_dim, int max_seg_len) {
  return (head_dim < 128 && max_seg_len > 1024) ? 256 : 128;
}

int attn_q_tile(bool bf16, int head_dim, int max_seg_len, int groups) {
  if (!bf16) {
    switch (head_dim) {
      case 8: case 16: case 32: case 64: case 72: case 80: case 96: case 128: return 64;
      default: return 0;
    }
  }
  if (groups < 0 || groups > 2) return 0;
  switch (head_dim) {
    case 32: case 64: case 72: case 80: case 96: case 128:
      return groups ? 128 * groups : bf16_q_rows(head_dim, max_seg_len);
    default: return 0;
  }
}

bool launch_attn_bf16(const AttnArgs& a, hipStream_t s) {
  if (a.num_work <= 0) return true;
  if (a.q_tile != 128 && a.q_tile != 256) return false;
  const bool wide = a.q_tile == 256;
  dim3 grid(a.num_work * a.num_heads);
  // The row of ones is used where the head dim leaves spare rows in its last 32-row block of
  // O^T (d = 72, 80: +3 % measured); for d = 32, 64, 96, 128 it would add a block of matrix
  // instructions and measured 2-7 % slower.
#define EPD_ATTN(DH)                                                                                     \
  case DH: {                                                                                             \
    constexpr bool sr = (DH % 32) != 0;                                                                  \
    if (wide) {                                                                                          \
      if constexpr (DH <= 64) hipLaunchKernelGGL((attn_bf16_kernel<DH, 2, 2, sr, 4>), grid, dim3(256), 0, s, a); \
      else hipLaunchKernelGGL((attn_bf16_kernel<DH, 1, 1, sr, 8>), grid, dim3(512), 0, s, a);          \
    } else {                                                                                             \
      hipLaunchKernelGGL((attn_bf16_kernel<DH, 1, (DH <= 64 ? 4 : 2), sr, 4>), grid, dim3(256), 0, s, a); \
    }                                                                                                    \
    return true;                                                                                         \
  }
  switch (a.head_dim) {
    EPD_ATTN(32);
    EPD_ATTN(64);
    EPD_ATTN(72);
    EPD_ATTN(80);
    EPD_ATTN(96);
    EPD_ATTN(128);
    default:
      return false;
  }
#undef EPD_ATTN
}

}  // namespace epd
