// bf16 GEMM family of the Encode-stage library (ViT forward, paper section 3.1, Eq. 1):
// patch embedding, QKV projection with rotary epilogue, attention output projection, the
// two MLP GEMMs and the merger projection all are  C[M,N] = A[M,K] * W[N,K]^T (+bias)  with
// different epilogues.  Written for gfx950: 64-lane waves, v_mfma_f32_16x16x32_bf16 (fp32
// accumulate; at equal flops this shape draws less power than the 32x32x16 one, and under the
// chip's power limit that is clock: +7 % on the large GEMMs with random operands, nothing on
// all-zero ones), operand tiles brought from global memory straight into LDS
// (global_load_lds_dwordx4, no register staging) in a two-stage ring.
//
// Tile scheme.  A block of WAVES_M x WAVES_N waves owns a BM x BN output tile; K advances in
// steps of BK.  Both operands are K-contiguous in memory ("NT" form), so one lane's MFMA
// operand (8 consecutive k of one row) is one 16-byte LDS read.  A direct-to-LDS load writes
// the 64 lanes' 16-byte chunks to consecutive LDS addresses, so rows cannot be padded;
// instead the chunk a lane fetches is chosen so that chunk c of row r lands in slot
// c ^ swz(r) of that row, which spreads the 16 rows read by one MFMA operand fetch over all
// bank groups.  Stage s+1 is in flight while stage s is multiplied; one barrier per K step.
//
// Accumulator orientation.  For a 16x16 MFMA result lane l holds column (l % 16) and rows
// 4*(l/16) + v, v = 0..3.  By default the W fragment is fed as the first operand, so "rows"
// are output columns n and the lane's column is a token m: every lane then owns runs of 4
// consecutive n of one token -- 16-byte fp32 / 8-byte bf16 pieces of a row, and the two
// members of a rotary pair (neighbouring n after the create-time reorder) share a lane.  For
// the V third of the QKV projection the operands are swapped, a lane owns 4 consecutive tokens
// of one n, and V is stored transposed ([channel][token]) for the attention kernel's second
// GEMM.
#include "epd_internal.h"

#include <algorithm>
#include <type_traits>

namespace epd {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;

#define EPD_GPTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define EPD_LPTR(p) ((__attribute__((address_space(3))) void*)(p))

__device__ __forceinline__ uint2 pack_bf16x4(float a, float b, float c, float d) {
  bf16x2 lo, hi;
  lo[0] = (__bf16)a; lo[1] = (__bf16)b; hi[0] = (__bf16)c; hi[1] = (__bf16)d;
  uint2 r;
  r.x = *(uint32_t*)&lo; r.y = *(uint32_t*)&hi;
  return r;
}

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

// x * Phi(x) with the Gaussian CDF written through its upper tail,
//   gelu(x) = max(x, 0) - |x| Q(|x|),   Q(a) = erfc(a / sqrt2) / 2 = 2^(a P(a) - 1),
// where P is a degree-5 polynomial fitted (weighted minimax, a in [0, 7.5]) to
// log2(erfc(a / sqrt2)) / a.  The logarithm of the tail is smooth, so one v_exp_f32 and six
// fused multiply-adds reach an absolute error below 2e-6 and a relative error below 1.5e-3 even
// where gelu is of order 1e-12 -- both far below the bf16 rounding of the stored result.
// Beyond a = 7.5 the tail term is below 1e-12 and the exponent is simply held.
__device__ __forceinline__ float gelu_erf_fast(float x) {
  const float a = fminf(fabsf(x), 7.5f);
  float p = fmaf(2.3815253741819458e-05f, a, -0.0006414791230697928f);
  p = fmaf(p, a, 0.007484599623650507f);
  p = fmaf(p, a, -0.05223089570546575f);
  p = fmaf(p, a, -0.459768916243223f);
  p = fmaf(p, a, -1.1509091680606687f);
  const float e = __builtin_amdgcn_exp2f(fmaf(p, a, -1.0f));
  return fmaf(-fabsf(x), e, fmaxf(x, 0.f));
}

__device__ __forceinline__ float gelu_tanh_fast(float x) {
  const float u = 0.79788456080286535588f * fmaf(0.044715f * x * x, x, x);
  const float e = __builtin_amdgcn_exp2f(2.0f * 1.44269504088896340736f * u);
  return x * (1.0f - __builtin_amdgcn_rcpf(1.0f + e));   // x * sigmoid(2u)
}

enum OutKind : int { OUT_BF16 = 0, OUT_F32 = 1 };

// Sum over aligned groups of G = 16 or 32 consecutive lanes; every lane of a group gets the sum.
template <int G> __device__ __forceinline__ float group_sum(float x) {
  static_assert(G == 16 || G == 32, "group size");
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xF, 0xF, true));   // quad_perm 1,0,3,2
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xF, 0xF, true));   // quad_perm 2,3,0,1
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x141, 0xF, 0xF, true));  // row_half_mirror
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x140, 0xF, 0xF, true));  // row_mirror
  if constexpr (G == 32)
    x += __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((int)((threadIdx.x ^ 16) & 63) * 4, __builtin_bit_cast(int, x)));
  return x;
}

// LDS beyond the operand stages: the rotary epilogue keeps the tile's cos / sin table there, up
// to 256 + QKV_TABLE_EXTRA bytes per token (head_dim 72 has 36 pairs of 8 bytes)
constexpr int QKV_TABLE_EXTRA = 32;
template <class T, int EPI> __host__ __device__ constexpr int lds_extra() { return EPI == 3 ? T::BM * QKV_TABLE_EXTRA : 0; }

template <int N> __device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Explicit LDS reads and counter waits (see the main loop of gemm_tile for why).
template <int OFF> __device__ __forceinline__ void ds_read_b128(bf16x8& d, uint32_t addr) {
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(d) : "v"(addr), "n"(OFF) : "memory");
}
template <int N, int STRIDE, int BASE, int I = 0> __device__ __forceinline__ void ds_read_rows(bf16x8* d, uint32_t addr) {
  if constexpr (I < N) {
    static_assert(BASE + I * STRIDE < 65536, "LDS offset field");
    ds_read_b128<BASE + I * STRIDE>(d[I], addr);
    ds_read_rows<N, STRIDE, BASE, I + 1>(d, addr);
  }
}
// wait until at most PENDING LDS reads of this wave are outstanding (they return in order),
// then tie the N fragments to the wait so that their consumers cannot be scheduled above it
// The compiler takes the result of an inline ds_read for valid at once: the ties keep the
// consumers behind the wait, and the scheduling barrier keeps any register copy the compiler
// makes for a tie behind it as well -- a copy hoisted above the wait reads a register the LDS
// has not filled yet (seen once, with a variant of the main loop; the generated code of every
// kernel is checked for such copies at build time, check_lds_waits.py).
template <int PENDING, int N, int N2> __device__ __forceinline__ void wait_lds_reads(bf16x8* f, bf16x8* f2) {
  asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(PENDING) : "memory");
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int i = 0; i < N; ++i) asm volatile("" : "+v"(f[i]));
#pragma unroll
  for (int i = 0; i < N2; ++i) asm volatile("" : "+v"(f2[i]));
}

// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>), unrolled at compile time
template <class F, int... I> __device__ __forceinline__ void static_for_seq(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F> __device__ __forceinline__ void static_for(F&& f) {
  static_for_seq(f, std::make_integer_sequence<int, N>{});
}

// Compile-time description of one kernel variant.
template <int BM_, int BN_, int BK_, int WAVES_M_, int WAVES_N_, int MINBLK_, int PARTS_>
struct Tile {
  static constexpr int BM = BM_, BN = BN_, BK = BK_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
  static constexpr int MINBLK = MINBLK_;
  static constexpr int NT = 64 * WAVES_M * WAVES_N;
  static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N, TM = WM / 32, TN = WN / 32;
  static constexpr int TM16 = WM / 16, TN16 = WN / 16;   // 16 x 16 MFMA blocks per wave tile
  static constexpr int PARTS = PARTS_;                   // parts the A blocks of a k step are multiplied in
  static constexpr int CPR = BK / 8;                     // 16-byte chunks per tile row
  static constexpr int LA = BM * CPR / NT, LW = BN * CPR / NT;   // load instructions per thread and stage
  static constexpr int STAGE_BYTES = (BM + BN) * BK * 2;
  // fp32 epilogue staging (residual add, fp32 outputs): the tile's columns in 2 passes, or 4
  // where two would not fit LDS
  static constexpr int EPI_PASSES = BM * (BN / 2 * 4 + 16) <= 136 * 1024 ? 2 : 4;
  static constexpr int EPI_BYTES_A = BM * (BN / EPI_PASSES * 4 + 16), EPI_BYTES_V = (BN / EPI_PASSES) * (BM * 4 + 16);
  static constexpr int LDS_BYTES = (2 * STAGE_BYTES > EPI_BYTES_A ? 2 * STAGE_BYTES : EPI_BYTES_A) > EPI_BYTES_V
                                       ? (2 * STAGE_BYTES > EPI_BYTES_A ? 2 * STAGE_BYTES : EPI_BYTES_A) : EPI_BYTES_V;
  static_assert(BK == 64, "BK: the main loop is written for two MFMA k steps of 32 per stage");
  static_assert((BM * CPR) % NT == 0 && (BN * CPR) % NT == 0, "tile / thread mismatch");
  static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile");
  // LDS has 64 banks of 4 bytes: a 16-byte-per-lane read is served 16 lanes (256 bytes) at a
  // time, so 16 consecutive rows must map to 16 different 16-byte columns modulo 256 bytes.
  __device__ static __forceinline__ int swz(int row) { return (row >> 1) & 7; }
};

template <class T, int EPI, int OUT, bool VMODE, bool GATHER, bool FAST>
__device__ __forceinline__ void gemm_tile(const GemmArgs& g, const int m0, const int n0, char* const lds) {
  constexpr int BM = T::BM, BN = T::BN, BK = T::BK, NT = T::NT, WM = T::WM, WN = T::WN, TM = T::TM, TN = T::TN;
  constexpr int CPR = T::CPR, LA = T::LA, LW = T::LW;
  constexpr int ROWB = BK * 2;               // bytes per tile row
  constexpr int A_BYTES = BM * ROWB, W_BYTES = BN * ROWB;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps LDS bases scalar
  const int wm = wave / T::WAVES_N, wn = wave % T::WAVES_N;
  const int l16 = lane & 15, g4 = lane >> 4;

  const char* zeros = (const char*)g.zeros;
  const int kcw = GATHER ? g.K / g.gather_n : g.K;

  // ---- per-thread load descriptors.  Load instruction `it` of a stage covers LDS chunks
  // it*NT + wave*64 + lane; chunk c is row c / CPR, slot c % CPR, and holds k-chunk
  // slot ^ swz(row) of that row.  One instruction covers RPP = NT / CPR rows (a multiple of
  // 16, so the swizzle of a lane's row is the same for every `it`).
  //   FAST (the caller guarantees that whole tiles of A and W may be read, also where they
  //   run past M or N, and K is a multiple of BK): the address is a wave-uniform row base,
  //   advanced with scalar arithmetic, plus ONE per-lane offset for all loads of an operand.
  //   Otherwise rows beyond M (or N) are clamped to the last valid row -- they only feed
  //   accumulators that are never stored -- and every load keeps its own per-lane offset.
  constexpr int RPP = NT / CPR;
  static_assert(RPP % 16 == 0, "rows per load instruction");
  const char* a_base_ptr = (const char*)g.A + (size_t)m0 * g.lda * 2;
  const int ldw = g.ldw ? g.ldw : g.K;
  const char* w_base_ptr = (const char*)g.W + (size_t)n0 * ldw * 2;
  constexpr int NOFF_A = FAST ? 1 : LA, NOFF_W = FAST ? 1 : LW;
  uint32_t a_off[NOFF_A], w_off[NOFF_W];
#pragma unroll
  for (int it = 0; it < NOFF_A; ++it) {
    const int c = it * NT + tid, row = c / CPR, col = (c % CPR) ^ T::swz(row);
    a_off[it] = (uint32_t)(FAST ? row : min(row, g.M - 1 - m0)) * (uint32_t)g.lda * 2u + col * 16;
  }
#pragma unroll
  for (int it = 0; it < NOFF_W; ++it) {
    const int c = it * NT + tid, row = c / CPR, col = (c % CPR) ^ T::swz(row);
    w_off[it] = (uint32_t)(FAST ? row : min(row, g.N - 1 - n0)) * (uint32_t)ldw * 2u + col * 16;
  }
  // first k of the chunk that load instruction `it` fetches (only the ragged-K and gather paths
  // need it, so it is recomputed there rather than kept in registers)
  auto chunk_k = [&](int it) {
    const int c = it * NT + tid, row = c / CPR;
    return ((c % CPR) ^ T::swz(row)) * 8;
  };

  // TAIL = the K step that may run past K (only the last one, only when K % BK != 0):
  // chunks at k >= K are fetched from a zero buffer instead.
  // LDS: [A stage 0 | A stage 1 | W stage 0 | W stage 1]
  auto issue = [&](auto TAIL, int stage, int k0) {
    constexpr bool tail = decltype(TAIL)::value;
    char* const sa = lds + stage * A_BYTES;
    char* const sw = lds + 2 * A_BYTES + stage * W_BYTES;
    const char* ab = a_base_ptr + (size_t)k0 * 2;
    const char* wb = w_base_ptr + (size_t)k0 * 2;
    // The per-lane offsets pass through an opaque copy here, so that their widening to 64 bits
    // stays next to the load: "scalar base + 32-bit lane offset" is then the load's own
    // addressing form.  Widened once ahead of the loop, every offset would occupy a register
    // pair for the whole loop and every load would need a 64-bit vector add in front of it.
    // (one copy per load: a shared one would let the adds be re-associated into a running
    // 64-bit vector address again)
    uint32_t ao[LA], wo[LW];
#pragma unroll
    for (int it = 0; it < LA; ++it) { ao[it] = a_off[FAST ? 0 : it]; asm volatile("" : "+v"(ao[it])); }
#pragma unroll
    for (int it = 0; it < LW; ++it) { wo[it] = w_off[FAST ? 0 : it]; asm volatile("" : "+v"(wo[it])); }
#pragma unroll
    for (int it = 0; it < LA; ++it) {
      const char* p;
      if constexpr (GATHER) {
        const int k = k0 + chunk_k(it);
        const int piece = min(k / kcw, g.gather_n - 1);
        const int row = min((it * NT + tid) / CPR, g.M - 1 - m0);
        const int src = g.gather[(size_t)(m0 + row) * g.gather_n + piece];
        p = (const char*)g.A + ((size_t)src * g.lda + (k - piece * kcw)) * 2;
      } else if constexpr (FAST) {
        p = (ab + (size_t)(it * RPP) * (size_t)g.lda * 2) + (size_t)ao[it];
      } else {
        p = ab + (size_t)ao[it];
      }
      if constexpr (tail) { if (k0 + chunk_k(it) >= g.K) p = zeros; }
      __builtin_amdgcn_global_load_lds(EPD_GPTR(p), EPD_LPTR(sa + (it * NT + wave * 64) * 16), 16, 0, 0);
    }
#pragma unroll
    for (int it = 0; it < LW; ++it) {
      const char* p;
      if constexpr (FAST) p = (wb + (size_t)(it * RPP) * (size_t)ldw * 2) + (size_t)wo[it];
      else p = wb + (size_t)wo[it];
      if constexpr (tail) { if (k0 + chunk_k(it) >= g.K) p = zeros; }
      __builtin_amdgcn_global_load_lds(EPD_GPTR(p), EPD_LPTR(sw + (it * NT + wave * 64) * 16), 16, 0, 0);
    }
  };
  // Folded RMSNorm (consumer side): scale of row m = rsqrt(mean of squares + eps), from the
  // per-segment sums the producing GEMM left.  Computed first, so that the loads complete in
  // the shadow of the main loop, and kept in LDS behind the stages and the staging area (the
  // barriers of the main loop make it visible to the epilogue).
  float* const row_scale = (float*)(lds + T::LDS_BYTES + lds_extra<T, EPI>());
  const bool scaled = g.stats_in != nullptr;
  // eight segments (hidden 1024): the loads are issued here, ahead of the first operand
  // loads, and only consumed after the first barrier
  static_assert(BM <= NT, "one row scale per thread");
  const bool scaled8 = scaled && g.stats_n == 8;
  float4 st_a = make_float4(0.f, 0.f, 0.f, 0.f), st_b = st_a;
  if (scaled8) {
    if (tid < BM) {
      const float4* sp = (const float4*)(g.stats_in + (size_t)min(m0 + tid, g.M - 1) * 8);
      st_a = sp[0]; st_b = sp[1];
    }
  } else if (scaled) {
    for (int r = tid; r < BM; r += NT) {
      const float* sp = g.stats_in + (size_t)min(m0 + r, g.M - 1) * g.stats_n;
      float ss = 0.f;
      for (int j = 0; j < g.stats_n; ++j) ss += sp[j];
      row_scale[r] = 1.0f / sqrtf(fmaf(ss, g.stats_inv_dim, g.stats_eps));
    }
  }

  // bf16 store / activation epilogue: its bias values (4 columns per 8-column group of the
  // lane) are fetched here, so that their latency passes in the shadow of the main loop; the
  // largest tile has no registers to spare for them and fetches them in the epilogue
  constexpr bool BF16_EPI = (EPI == EPI_STORE || EPI == EPI_GELU) && OUT == OUT_BF16 && !VMODE;
  constexpr bool BIAS_PRE = BF16_EPI && BM * BN <= 256 * 256;
  [[maybe_unused]] uint2 bb[TN][2];
  auto load_bias = [&]() {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const int nb = n0 + wn * WN + j * 32 + c * 16 + g4 * 4;
        bb[j][c] = (g.bias && nb < g.N) ? *(const uint2*)((const uint16_t*)g.bias + nb) : make_uint2(0u, 0u);   // N is a multiple of 4
      }
  };
  if constexpr (BIAS_PRE) load_bias();

  const int nk = (g.K + BK - 1) / BK;
  const bool ragged_k = (g.K % BK) != 0;
  auto issue_step = [&](int stage, int kt) {      // kt < nk
    if constexpr (FAST) {
      issue(std::false_type{}, stage, kt * BK);
    } else {
      if (ragged_k && kt == nk - 1) issue(std::true_type{}, stage, kt * BK);
      else issue(std::false_type{}, stage, kt * BK);
    }
  };

  // acc[i][j][q]: the 32 x 32 block (i, j) of the wave tile as four 16 x 16 MFMA results,
  // q = 2 * (token half) + (column half)
  f32x4 acc[TM][TN][4];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[i][j][q][v] = 0.f;

  // ---- LDS fragment reads.  Issued as explicit ds_read_b128 so that their order against the
  // direct-to-LDS loads and the waits below is exactly the one written here (a compiler-
  // visible LDS read that follows a direct-to-LDS load in program order gets a full wait for
  // that load inserted in front of it, which would serialise the two-stage ring).
  // One fragment = 16 rows x 32 k: lane (l16, g4) reads k chunk 4*ks + g4 of row blk*16 + l16;
  // multiples of 16 keep swz(row) = swz(l16).  A stage is multiplied in 2 * P slices,
  // slice sl = (k step ks = sl / P, part p = sl % P of the A blocks): slice (ks, 0) needs the
  // TN16 W fragments of the k step and the first AP A fragments, the others the next AP A
  // fragments.  W fragments alternate between two buffers by k step, A fragments by slice.
  constexpr int TM16 = T::TM16, TN16 = T::TN16, P = T::PARTS, AP = TM16 / P, NSL = 2 * P;
  static_assert(TM16 % P == 0 && TN16 + AP <= 15, "slices / LDS counter");
  constexpr bool LATE_REFILL = TM * TN <= 4;
  const uint32_t lds0 = (uint32_t)(size_t)EPD_LPTR(lds);
  // Address of k step 1 = address of k step 0 with bit 6 flipped (chunk slot bit 2; the row
  // base has a zero there); stage and 16-row block go into the instruction's offset field.
  const uint32_t a_rd0 = lds0 + (wm * WM + l16) * ROWB + ((g4 ^ T::swz(l16)) * 16);
  const uint32_t w_rd0 = lds0 + 2 * A_BYTES + (wn * WN + l16) * ROWB + ((g4 ^ T::swz(l16)) * 16);
  bf16x8 fw[2][TN16], fa[2][AP];
  auto read_slice = [&](auto SL, auto ST) {
    constexpr int sl = decltype(SL)::value, st = decltype(ST)::value, ks = sl / P, p = sl % P;
    if constexpr (p == 0) ds_read_rows<TN16, 16 * ROWB, st * W_BYTES>(&fw[ks][0], w_rd0 ^ (uint32_t)(ks * 64));
    ds_read_rows<AP, 16 * ROWB, st * A_BYTES + p * AP * 16 * ROWB>(&fa[sl & 1][0], a_rd0 ^ (uint32_t)(ks * 64));
  };
  // wait until at most the reads of the next slice are outstanding (none with DRAIN: every
  // read of the wave has returned), then tie the slice's fragments to the wait
  auto wait_slice = [&](auto SL, auto DRAIN) {
    constexpr int sl = decltype(SL)::value, ks = sl / P, p = sl % P;
    constexpr int next_reads = ((sl + 1) % P == 0 ? TN16 : 0) + AP;
    wait_lds_reads<(decltype(DRAIN)::value ? 0 : next_reads), AP, (p == 0 ? TN16 : 0)>(&fa[sl & 1][0], &fw[ks][0]);
  };
  auto mfmas = [&](auto SL) {
    constexpr int sl = decltype(SL)::value, ks = sl / P, p = sl % P;
    // consecutive MFMAs keep their first operand: measured ~7% faster than alternating it
    if constexpr (VMODE) {
#pragma unroll
      for (int t = 0; t < AP; ++t)
#pragma unroll
        for (int w = 0; w < TN16; ++w) {
          const int a16 = p * AP + t;
          acc[a16 >> 1][w >> 1][(a16 & 1) * 2 + (w & 1)] =
              __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[sl & 1][t], fw[ks][w], acc[a16 >> 1][w >> 1][(a16 & 1) * 2 + (w & 1)], 0, 0, 0);
        }
    } else {
#pragma unroll
      for (int w = 0; w < TN16; ++w)
#pragma unroll
        for (int t = 0; t < AP; ++t) {
          const int a16 = p * AP + t;
          acc[a16 >> 1][w >> 1][(a16 & 1) * 2 + (w & 1)] =
              __builtin_amdgcn_mfma_f32_16x16x32_bf16(fw[ks][w], fa[sl & 1][t], acc[a16 >> 1][w >> 1][(a16 & 1) * 2 + (w & 1)], 0, 0, 0);
        }
    }
  };
  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;
  using LAST = std::integral_constant<int, NSL - 1>;

  // Residual rows this thread updates in the epilogue (EPI_RESIDUAL, where its whole share is
  // at most 16 float4): fetched behind the last stage hand-over, so that the read of the
  // residual stream overlaps the last K step instead of standing at the head of the epilogue.
  // Rows and columns beyond the matrix are clamped (what they fetch is not used).
  constexpr int E_HALF = BN / T::EPI_PASSES, E_LPR4 = E_HALF / 4, E_RPS = NT / E_LPR4, E_SW = BM / E_RPS;
  constexpr bool PREF = EPI == EPI_RESIDUAL && !VMODE && T::EPI_PASSES * E_SW <= 16;
  [[maybe_unused]] float4 xpre[PREF ? T::EPI_PASSES * E_SW : 1];
  auto prefetch_resid = [&]() {
    if constexpr (PREF) {
#pragma unroll
      for (int h = 0; h < T::EPI_PASSES; ++h)
#pragma unroll
        for (int sw = 0; sw < E_SW; ++sw) {
          const int m = min(m0 + sw * E_RPS + tid / E_LPR4, g.M - 1);
          const int n = min(n0 + h * E_HALF + (tid % E_LPR4) * 4, g.N - 4);
          xpre[h * E_SW + sw] = *(const float4*)(g.resid + (size_t)m * g.ldr + n);
        }
    }
  };

  // ---- main loop: two LDS stages.  The hand-over to the next stage happens before the last
  // slice of the current stage is multiplied: wait for the own loads of stage s^1, barrier
  // (everybody's loads landed, everybody finished reading stage s), refill stage s with K step
  // kt+2, start reading stage s^1 -- and only then issue the MFMAs of the last slice, which
  // cover the barrier and the LDS latency.  Every load has one full K step to land.
  issue_step(0, 0);
  wait_vmcnt<0>();
  __builtin_amdgcn_s_barrier();
  if (scaled8 && tid < BM) {
    const float ss = ((st_a.x + st_a.y) + (st_a.z + st_a.w)) + ((st_b.x + st_b.y) + (st_b.z + st_b.w));
    row_scale[tid] = 1.0f / sqrtf(fmaf(ss, g.stats_inv_dim, g.stats_eps));
  }
  if (nk > 1) issue_step(1, 1);
  read_slice(I0{}, I0{});

  auto step = [&](auto S, int kt) {
    constexpr int s = decltype(S)::value;
    using SN = std::integral_constant<int, s ^ 1>;
    // the fragments of slice sl+1 are requested before slice sl is multiplied
    static_for<NSL - 1>([&](auto SL) {
      read_slice(std::integral_constant<int, decltype(SL)::value + 1>{}, S);
      wait_slice(SL, std::false_type{});
      mfmas(SL);
    });
    // last slice: stage hand-over first
    if (kt + 1 < nk) {
      wait_vmcnt<0>();
      wait_slice(LAST{}, std::true_type{});
      __builtin_amdgcn_s_barrier();
      if constexpr (!LATE_REFILL) {
        if (kt + 2 < nk) issue_step(s, kt + 2);
      }
      read_slice(I0{}, SN{});
      if (kt + 2 >= nk) prefetch_resid();          // last hand-over: no operand load follows
    } else {
      wait_slice(LAST{}, std::true_type{});
    }
    mfmas(LAST{});
    if constexpr (LATE_REFILL) {
      // small wave tiles: the refill of stage s is issued behind the queued MFMAs, so the
      // address arithmetic and load instructions run in their shadow (pinning this order
      // costs registers, which the large wave tiles do not have)
      __builtin_amdgcn_sched_barrier(0);
      if (kt + 2 < nk) issue_step(s, kt + 2);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  for (int kt = 0; kt < nk; kt += 2) {
    step(I0{}, kt);
    if (kt + 1 < nk) step(I1{}, kt + 1);
  }
  if (nk == 1) prefetch_resid();

  // ------------------------------------------------------------------ epilogue
  // The accumulators go through LDS (the operand stages are dead by now) so that global
  // memory sees row-contiguous accesses: straight from the MFMA layout every store
  // instruction would touch 32 different rows with 16 bytes each.  Four forms follow: the V
  // tiles of QKV (transposed), bf16 store / activation and Q | K with rotary (passes over row
  // blocks, described where they stand), and the general one, used by the residual add and
  // fp32 outputs: two or four passes, each staging a slice of the tile's columns as fp32 (BM
  // rows x BN/passes floats, rows padded by 16 bytes); then every group of 16 or 32 lanes owns
  // one row and a lane owns 4 consecutive columns, which is where bias and the residual add
  // are applied.
  constexpr int NPASS = T::EPI_PASSES;
  constexpr int HALF = BN / NPASS;                    // columns per pass
  constexpr int WPH = T::WAVES_N / NPASS;             // wave columns per pass
  static_assert(T::WAVES_N % NPASS == 0 && HALF % 32 == 0, "epilogue passes");
  const uint16_t* bias = (const uint16_t*)g.bias;
  wait_vmcnt<0>();
  if constexpr (VMODE) {
    // The MFMA operands are swapped for these tiles, so a lane holds 4 consecutive tokens of
    // one channel: scale and bias are applied there and the bf16 values staged transposed,
    // ET[channel][token], the whole tile at once where it fits and in two channel halves where
    // not; a lane then takes 8 consecutive tokens (one 16-byte store) of a channel row.
    constexpr int ROWV = BM * 2 + 16;
    constexpr int NPV = BN * ROWV <= T::LDS_BYTES ? 1 : 2;          // passes
    constexpr int CPV = BN / NPV;                                   // channels per pass
    static_assert(CPV * ROWV <= T::LDS_BYTES && CPV % WN == 0, "transposed staging area");
    uint16_t* vt = (uint16_t*)g.vt;
    // thread coordinates derived afresh (through an opaque copy of the thread id): nothing of
    // this epilogue's index arithmetic is then computed ahead of the main loop and kept in
    // registers across it, where the largest tile has none to spare
    int tid_v = threadIdx.x;
    asm volatile("" : "+v"(tid_v));
    const int tid = tid_v, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / T::WAVES_N, wn = wave % T::WAVES_N, l16 = lane & 15, g4 = lane >> 4;
    // BM tokens per channel row: BM/8 lanes per row, 8 tokens per lane
    constexpr int LPRV = BM / 8, RPS = NT / LPRV;        // threads beyond RPS whole rows idle
    const int tl = (tid % LPRV) * 8;
    const int m = tid < RPS * LPRV ? m0 + tl : g.M;
    int4 vc0 = make_int4(0, 0, 0, 0), vc1 = make_int4(0, 0, 0, 0);
    const bool full = m + 7 < g.M;
    if (full) { vc0 = *(const int4*)(g.vcol + m); vc1 = *(const int4*)(g.vcol + m + 4); }
    const bool fast = full && (vc1.w - vc0.x == 7) && ((vc0.x & 7) == 0);
#pragma unroll
    for (int ps = 0; ps < NPV; ++ps) {
      __syncthreads();
      if ((wn * WN) / CPV == ps) {
#pragma unroll
        for (int jc = 0; jc < 2 * TN; ++jc) {
          const int j = jc >> 1, c = jc & 1;
          const int chl = wn * WN + jc * 16 + l16;       // channel inside the tile
          const float bv = (bias && n0 + chl < g.N) ? bf16_bits_to_float(bias[n0 + chl]) : 0.f;
#pragma unroll
          for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int t = 0; t < 2; ++t) {
              const int ml = wm * WM + i * 32 + t * 16 + g4 * 4;
              const f32x4 a = acc[i][j][2 * t + c];
              float4 rs = make_float4(1.f, 1.f, 1.f, 1.f);
              if (scaled) rs = *(const float4*)(row_scale + ml);
              *(uint2*)(lds + (chl - ps * CPV) * ROWV + ml * 2) =
                  pack_bf16x4(fmaf(a[0], rs.x, bv), fmaf(a[1], rs.y, bv), fmaf(a[2], rs.z, bv), fmaf(a[3], rs.w, bv));
            }
        }
      }
      __syncthreads();
      for (int r = tid / LPRV; r < CPV; r += RPS) {
        const int n = n0 + ps * CPV + r;
        if (n >= g.N || m >= g.M) continue;
        const uint4 p = *(const uint4*)(lds + r * ROWV + tl * 2);
        uint16_t* vrow = vt + (size_t)(n - g.qk_cols) * g.vt_stride;
        if (fast) {
          *(uint4*)(vrow + vc0.x) = p;
        } else {
          const uint32_t w[4] = {p.x, p.y, p.z, p.w};
          for (int t = 0; t < 8 && m + t < g.M; ++t) vrow[g.vcol[m + t]] = (uint16_t)(w[t >> 1] >> ((t & 1) * 16));
        }
      }
    }
  } else if constexpr ((EPI == EPI_STORE || EPI == EPI_GELU) && OUT == OUT_BF16) {
    // bf16 output with a per-element epilogue that needs nothing but the element and its
    // column: scale, bias and activation are applied in the MFMA layout (a lane holds 4
    // consecutive columns of one token) and the finished bf16 values are staged through LDS to
    // leave as 16-byte pieces of whole rows.  The passes split the tile by rows: pass i takes
    // row block i of every wave (32 rows per wave row, all BN columns), so every wave -- every
    // SIMD -- does a share of the activation arithmetic in every pass, and a row leaves as
    // BN * 2 contiguous bytes.  Two staging buffers alternate, which leaves one barrier per
    // pass: a buffer is rewritten two passes later, behind the barrier of the pass between.
    constexpr int SR = T::WAVES_M * 32;                // rows per pass
    constexpr int ROWO = BN * 2 + 16;                  // padded: 16 consecutive rows hit 16 different bank groups
    constexpr int BUF = SR * ROWO;
    constexpr int CPRO = BN / 8, RPSO = NT / CPRO;     // 16-byte chunks per row, rows per sweep
    static_assert(2 * BUF <= T::LDS_BYTES && SR % RPSO == 0 && NT % CPRO == 0, "bf16 staging area");
    uint16_t* const outp = (uint16_t*)g.out;
    const int c8 = (tid % CPRO) * 8;
    const int n = n0 + c8;
    const bool vec = (g.ldo % 8 == 0) && (((size_t)outp & 15) == 0) && n + 8 <= g.N;
    if constexpr (!BIAS_PRE) load_bias();
    __syncthreads();                                   // the operand stages are dead from here on
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      char* const buf = lds + (i & 1) * BUF;
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const float rs = scaled ? row_scale[wm * WM + i * 32 + t * 16 + l16] : 1.0f;
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int c = 0; c < 2; ++c) {
            const int nl = wn * WN + j * 32 + c * 16 + g4 * 4;       // column inside the tile
            const f32x4 a = acc[i][j][2 * t + c];
            const float b0 = bf16_bits_to_float(bb[j][c].x & 0xffff), b1 = bf16_bits_to_float(bb[j][c].x >> 16);
            const float b2 = bf16_bits_to_float(bb[j][c].y & 0xffff), b3 = bf16_bits_to_float(bb[j][c].y >> 16);
            float v0 = fmaf(a[0], rs, b0), v1 = fmaf(a[1], rs, b1), v2 = fmaf(a[2], rs, b2), v3 = fmaf(a[3], rs, b3);
            if constexpr (EPI == EPI_GELU) {
              if (g.act == 0) { v0 = gelu_erf_fast(v0); v1 = gelu_erf_fast(v1); v2 = gelu_erf_fast(v2); v3 = gelu_erf_fast(v3); }
              else { v0 = gelu_tanh_fast(v0); v1 = gelu_tanh_fast(v1); v2 = gelu_tanh_fast(v2); v3 = gelu_tanh_fast(v3); }
            }
            *(uint2*)(buf + (wm * 32 + t * 16 + l16) * ROWO + nl * 2) = pack_bf16x4(v0, v1, v2, v3);
          }
      }
      __syncthreads();
      if (n < g.N) {
#pragma unroll
        for (int sw = 0; sw < SR / RPSO; ++sw) {
          const int r = sw * RPSO + tid / CPRO;
          const int m = m0 + (r / 32) * WM + i * 32 + (r % 32);
          if (m >= g.M) continue;
          const uint4 v = *(const uint4*)(buf + r * ROWO + c8 * 2);
          uint16_t* dst = outp + (size_t)m * g.ldo + n;
          if (vec) {
            *(uint4*)dst = v;
          } else {
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
            for (int t = 0; t < 8 && n + t < g.N; ++t) dst[t] = (uint16_t)(w[t >> 1] >> ((t & 1) * 16));
          }
        }
      }
    }
  } else if constexpr (EPI == EPI_QKV) {
    // Q | K columns with rotary: the passes split the tile by rows, not by columns.  Pass i
    // stages row block i of every wave (32 rows per wave row, all BN columns, fp32), so all
    // waves write at once and a wave then reads and stores whole rows (BN * 2 bytes contiguous
    // in memory).  The cos / sin entries of the tile's tokens are one contiguous slab of the
    // table; it is copied into LDS behind the staging area by direct-to-LDS loads issued before
    // the first pass is staged, and every pass reads its entries from there (fetched from
    // memory per pass, their latency was more than half of this epilogue).  Staging rows are
    // unpadded and swizzled instead, 16-byte chunk c of row r at chunk c ^ (r % 16): staging
    // plus a table of up to 256 + QKV_TABLE_EXTRA bytes per token then fill the operand stages
    // exactly.  Larger tables (head_dim > 72) are read from memory.
    constexpr int SR = T::WAVES_M * 32;                // rows per pass
    constexpr int ROWE = BN * 4;
    constexpr int STG = SR * ROWE;
    constexpr int LPR4 = BN / 4, RPS = NT / LPR4;      // lanes per row (4 columns each), rows per sweep
    static_assert(STG <= T::LDS_BYTES && SR % RPS == 0 && NT % LPR4 == 0 && LPR4 >= 16, "row-split staging");
    const int cl = (tid % LPR4) * 4;
    const int n = n0 + cl;                             // N is a multiple of 4: all or nothing
    float b0 = 0.f, b1 = 0.f, b2 = 0.f, b3 = 0.f;
    if (bias && n < g.N) {
      const uint2 bb = *(const uint2*)(bias + n);
      b0 = bf16_bits_to_float(bb.x & 0xffff); b1 = bf16_bits_to_float(bb.x >> 16);
      b2 = bf16_bits_to_float(bb.y & 0xffff); b3 = bf16_bits_to_float(bb.y >> 16);
    }
    const int pr = (n % g.head_dim) >> 1;              // even: two pairs = one 16-byte entry
    const int trb = g.rot_pairs * 8;                   // table bytes per token
    const bool tab_lds = g.rot != nullptr && STG + BM * trb <= T::LDS_BYTES + lds_extra<T, EPI>();
    const char* const tab = lds + STG;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      __syncthreads();
      if (i == 0 && tab_lds) {
        // BM * trb bytes from row m0 of the table, 16 bytes per lane, a wave fills 1 KB of LDS
        // per instruction; rows past M are never used: their chunks re-read the last valid one
        const char* src = (const char*)g.rot + (size_t)m0 * trb;
        const long last = (long)(g.M - m0) * trb - 16;
        for (int c0 = wave * 64; c0 < BM * (trb / 16); c0 += NT)
          __builtin_amdgcn_global_load_lds(EPD_GPTR(src + min((long)(c0 + lane) * 16, last)), EPD_LPTR(tab + c0 * 16), 16, 0, 0);
      }
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int sr = wm * 32 + (q >> 1) * 16 + l16;
          const int ch = (wn * WN + j * 32 + (q & 1) * 16) / 4 + g4;
          const f32x4 a = acc[i][j][q];
          *(float4*)(lds + sr * ROWE + (ch ^ (sr & 15)) * 16) = make_float4(a[0], a[1], a[2], a[3]);
        }
      if (i == 0) wait_vmcnt<0>();
      __syncthreads();
      if (n < g.N) {
        // fully unrolled so that the LDS reads of all sweeps are in flight together
#pragma unroll
        for (int sw = 0; sw < SR / RPS; ++sw) {
          const int r = sw * RPS + tid / LPR4;
          const int ml = (r / 32) * WM + i * 32 + (r % 32);
          const int m = m0 + ml;
          if (m >= g.M) continue;
          const float4 e = *(const float4*)(lds + r * ROWE + (((tid % LPR4) ^ (r & 15)) * 16));
          const float rs = scaled ? row_scale[ml] : 1.0f;
          float v0 = fmaf(e.x, rs, b0), v1 = fmaf(e.y, rs, b1), v2 = fmaf(e.z, rs, b2), v3 = fmaf(e.w, rs, b3);
          if (g.rot) {
            const float4 cs = tab_lds ? *(const float4*)(tab + ml * trb + pr * 8)
                                      : *(const float4*)(g.rot + (size_t)m * g.rot_pairs + pr);
            const float r0 = v0 * cs.x - v1 * cs.y, r1 = v0 * cs.y + v1 * cs.x;
            const float r2 = v2 * cs.z - v3 * cs.w, r3 = v2 * cs.w + v3 * cs.z;
            v0 = r0; v1 = r1; v2 = r2; v3 = r3;
          }
          // the softmax scale (in log2 units) rides on Q: one rounding of q * scale instead of
          // a multiply per score in the attention kernel
          if (n < g.q_cols) { v0 *= g.q_scale; v1 *= g.q_scale; v2 *= g.q_scale; v3 *= g.q_scale; }
          *(uint2*)((uint16_t*)g.out + (size_t)m * g.ldo + n) = pack_bf16x4(v0, v1, v2, v3);
        }
      }
    }
  } else {
    constexpr int ROWE = HALF * 4 + 16;
    constexpr int LPR4 = HALF / 4, RPS = NT / LPR4;    // lanes per row (4 columns each), rows per sweep
    static_assert(BM % RPS == 0, "sweeps");
    const int cl = (tid % LPR4) * 4;                   // first of the lane's 4 columns inside the half
    static_assert(HALF == 64 || HALF == 128, "sum-of-squares segments are 128 columns");
    [[maybe_unused]] float seg_ss[BM / RPS];
#pragma unroll
    for (int h = 0; h < NPASS; ++h) {
      __syncthreads();
      if (wn / WPH == h) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
          for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const int ml = wm * WM + i * 32 + (q >> 1) * 16 + l16;
              const int nl = (wn % WPH) * WN + j * 32 + (q & 1) * 16 + g4 * 4;
              const f32x4 a = acc[i][j][q];
              *(float4*)(lds + ml * ROWE + nl * 4) = make_float4(a[0], a[1], a[2], a[3]);
            }
        }
      }
      __syncthreads();
      const int n = n0 + h * HALF + cl;
      if (n >= g.N) continue;                          // N is a multiple of 4: all or nothing
      float b0 = 0.f, b1 = 0.f, b2 = 0.f, b3 = 0.f;
      if (bias) {
        const uint2 bb = *(const uint2*)(bias + n);
        b0 = bf16_bits_to_float(bb.x & 0xffff); b1 = bf16_bits_to_float(bb.x >> 16);
        b2 = bf16_bits_to_float(bb.y & 0xffff); b3 = bf16_bits_to_float(bb.y >> 16);
      }
      // fully unrolled so that the residual loads / LDS reads of all sweeps are in flight together
#pragma unroll
      for (int sw = 0; sw < BM / RPS; ++sw) {
        const int r = sw * RPS + tid / LPR4;
        const int m = m0 + r;
        if (m >= g.M) continue;
        const float4 e = *(const float4*)(lds + r * ROWE + cl * 4);
        const float rs = scaled ? row_scale[r] : 1.0f;
        float v0 = fmaf(e.x, rs, b0), v1 = fmaf(e.y, rs, b1), v2 = fmaf(e.z, rs, b2), v3 = fmaf(e.w, rs, b3);
        if constexpr (EPI == EPI_GELU) {
          if (g.act == 0) { v0 = gelu_erf_fast(v0); v1 = gelu_erf_fast(v1); v2 = gelu_erf_fast(v2); v3 = gelu_erf_fast(v3); }
          else { v0 = gelu_tanh_fast(v0); v1 = gelu_tanh_fast(v1); v2 = gelu_tanh_fast(v2); v3 = gelu_tanh_fast(v3); }
        }
        if constexpr (EPI == EPI_RESIDUAL) {
          float4* xp = (float4*)(g.resid + (size_t)m * g.ldr + n);
          float4 x;
          if constexpr (PREF) x = xpre[h * E_SW + sw];
          else x = *xp;
          x.x += v0; x.y += v1; x.z += v2; x.w += v3;
          *xp = x;
          // folded RMSNorm (producer side): the raw rows in bf16 for the next GEMM, and their
          // sums of squares per 128-column segment (HALF = 64: two passes make one segment)
          if (g.xb) *(uint2*)((uint16_t*)g.xb + (size_t)m * g.ldxb + n) = pack_bf16x4(x.x, x.y, x.z, x.w);
          if (g.stats_out) {
            const float ss = group_sum<LPR4>(fmaf(x.x, x.x, fmaf(x.y, x.y, fmaf(x.z, x.z, x.w * x.w))));
            if constexpr (HALF == 128) {
              if ((tid % LPR4) == 0) g.stats_out[(size_t)m * g.stats_n + (n0 + h * HALF) / 128] = ss;
            } else {
              seg_ss[sw] = (h % 2 == 0) ? ss : seg_ss[sw] + ss;
              if (h % 2 == 1 && (tid % LPR4) == 0) g.stats_out[(size_t)m * g.stats_n + (n0 + (h / 2) * 128) / 128] = seg_ss[sw];
            }
          }
        } else if constexpr (OUT == OUT_F32) {
          *(float4*)((float*)g.out + (size_t)m * g.ldo + n) = make_float4(v0, v1, v2, v3);
        } else {
          *(uint2*)((uint16_t*)g.out + (size_t)m * g.ldo + n) = pack_bf16x4(v0, v1, v2, v3);
        }
      }
    }
  }
}

// Consecutive hardware block ids go to different XCDs (8 per chip, each with its own 4 MB
// L2).  Remap so that every XCD walks a contiguous range of tile numbers, and number the tiles
// in groups of `group_m` row tiles swept column by column: the tiles an XCD runs at the same
// time then form a compact rectangle whose A panels stay in its L2 while W panels stream
// through once, instead of every XCD re-reading all of W for every row of tiles.
__device__ __forceinline__ int xcd_remap(int bid, int nblocks) {
  const int q = nblocks >> 3, r = nblocks & 7;
  const int xcd = bid & 7, idx = bid >> 3;
  return xcd * q + min(xcd, r) + idx;
}

__device__ __forceinline__ void tile_coords(int t, int tiles_m, int tiles_n, int group_m, int& tm, int& tn) {
  const int per_group = group_m * tiles_n;
  const int grp = t / per_group, local = t - grp * per_group;
  const int first = grp * group_m;
  const int rows = min(group_m, tiles_m - first);
  tn = local / rows;
  tm = first + (local - tn * rows);
}

// TAG changes nothing in the code: it gives the two residual GEMMs of a block (attention output
// projection, second MLP GEMM) kernel names of their own, so that a profile lists them apart.
template <class T, int EPI, int OUT, bool GATHER, bool FAST, int TAG>
__global__ __launch_bounds__(T::NT, T::MINBLK) void gemm_bf16_kernel(GemmArgs g) {
  // + room for a wider rotary table (QKV epilogue) + per-row scales of the epilogue
  __shared__ __attribute__((aligned(1024))) char lds[T::LDS_BYTES + lds_extra<T, EPI>() + T::BM * 4];
  const int tiles_n = (g.N + T::BN - 1) / T::BN, tiles_m = (g.M + T::BM - 1) / T::BM;
  int tm, tn;
  tile_coords(xcd_remap(blockIdx.x, gridDim.x), tiles_m, tiles_n, g.group_m, tm, tn);
  const int m0 = tm * T::BM, n0 = tn * T::BN;
  if constexpr (EPI == EPI_QKV) {
    if (n0 >= g.qk_cols) {
      gemm_tile<T, EPI, OUT, true, false, FAST>(g, m0, n0, lds);
      return;
    }
  }
  gemm_tile<T, EPI, OUT, false, GATHER, FAST>(g, m0, n0, lds);
}

static int num_cus() {
  static int n = [] {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0)
      v = 256;
    return v;
  }();
  return n;
}

template <class T, int EPI, int OUT, bool GATHER>
static void launch_cfg(const GemmArgs& g, hipStream_t s) {
  const int tiles_m = (g.M + T::BM - 1) / T::BM, tiles_n = (g.N + T::BN - 1) / T::BN;
  GemmArgs a = g;
  if (a.group_m <= 0) {
    // keep the A panels of one group (group_m x BM rows x K) within about 2 MB of the 4 MB L2
    const long panel = (long)T::BM * g.K * 2;
    a.group_m = (int)std::max(1L, std::min((long)tiles_m, (2L << 20) / std::max(panel, 1L)));
    // Long K (panels beyond the cache) and a wide output: the 32 tiles an XCD runs at a time still
    // advance through K together, so what has to stay cached is their current K window, not whole
    // panels.  Four row tiles per group make that set 4 x 8 tiles (12 operand panels) instead of
    // 1 x 32 (33 panels): +5 % on 32768 x 12800 x 3200 and 32768 x 9600 x 3200; narrow outputs
    // (13 column tiles) measured best with the panel rule alone.
    if (tiles_n >= 24) a.group_m = std::max(a.group_m, 4);
    // Few rows against a large weight matrix (the merger projection): with row groups every
    // XCD streams all of W.  When the whole grid runs in at most two rounds, number the tiles
    // column by column instead, so that an XCD owns a block of columns: W is then fetched
    // once in total and the (smaller) A once per XCD.
    const long blocks = (long)T::MINBLK * (g.compute_units > 0 ? g.compute_units : num_cus());
    if ((long)g.N > 2L * g.M && (long)tiles_m * tiles_n <= 2 * blocks) a.group_m = tiles_m;
  }
  a.group_m = std::min(a.group_m, tiles_m);
  if constexpr (!GATHER) {
    if (g.overread_ok && g.K % T::BK == 0) {
      if (EPI == EPI_RESIDUAL && g.name_tag == 1)
        hipLaunchKernelGGL((gemm_bf16_kernel<T, EPI, OUT, false, true, (EPI == EPI_RESIDUAL ? 1 : 0)>), dim3(tiles_m * tiles_n), dim3(T::NT), 0, s, a);
      else
        hipLaunchKernelGGL((gemm_bf16_kernel<T, EPI, OUT, false, true, 0>), dim3(tiles_m * tiles_n), dim3(T::NT), 0, s, a);
      return;
    }
  }
  hipLaunchKernelGGL((gemm_bf16_kernel<T, EPI, OUT, GATHER, false, 0>), dim3(tiles_m * tiles_n), dim3(T::NT), 0, s, a);
}

//            BM   BN  BK  WM WN MINBLK PARTS
using T0 = Tile<256, 256, 64, 2, 4, 1, 4>;   // 8 waves, 128x64 wave tiles, 128 KB LDS, one block per CU
using T2 = Tile<256, 128, 64, 2, 2, 1, 4>;   // 4 waves, 128x64 wave tiles, 96 KB LDS
using T4 = Tile<128, 128, 64, 2, 2, 2, 4>;   // 4 waves, 64x64 wave tiles, 64 KB LDS, two blocks per CU
using T5 = Tile<320, 256, 64, 2, 4, 1, 5>;   // 8 waves, 160x64 wave tiles, 144 KB LDS, one block per CU

// Tile choice.  Both large tiles run one block per compute unit, so an output whose number of
// tiles is not a multiple of the unit count pays a whole tile time for its last, partial round,
// and nothing hides their epilogues.  The 128 x 128 tile runs two blocks per unit (the epilogue of
// one hides behind the main loop of the other) and quantises four times finer, but its main loop
// is the slowest.  The 320 x 256 tile moves the fewest operand bytes per flop.  A launch is priced
// by a model fitted to launch times measured INSIDE encoder calls (where the chip sits at its
// power limit; loops of one GEMM alone rank the tiles differently): the time of one round of
// blocks is, per 256 x 256 of output area,  alpha * K / 1024 + eps[epilogue]  microseconds
// (32768-token and 73896-token batches, K = 1024 ... 12800; it reproduces the measured launches
// of the 6272-token batch as well):
//                  alpha   eps: store / GELU   residual add   QKV + rotary
//   256 x 256      22.6        13.2               39.4            21.9
//   320 x 256      21.8        11.7               39.4            24.8
//   128 x 128      32.8         4.6               23.8            19.6
// So the small tile wins short-K GEMMs with a heavy epilogue (the attention output projection at
// hidden 1024), the 320 x 256 tile gains with short K and on grids where it needs fewer rounds,
// and at K >= 3200 the two large tiles are equal.
struct TileShape { int bm, bn, blocks, cfg; double alpha, eps[4]; };   // eps indexed by Epilogue
constexpr TileShape kShape256 = {256, 256, 1, 0, 22.6, {13.2, 13.2, 39.4, 21.9}};
constexpr TileShape kShape320 = {320, 256, 1, 5, 21.8, {11.7, 11.7, 39.4, 24.8}};
constexpr TileShape kShape128 = {128, 128, 2, 4, 32.8, {4.6, 4.6, 23.8, 19.6}};
constexpr double kSecondLaunch = 4.0;      // what a second launch of the same GEMM adds (gap + ramp), same unit

static double tile_cost(int M, int N, int K, int epi, const TileShape& t, long cus) {
  const long tiles = (long)((M + t.bm - 1) / t.bm) * ((N + t.bn - 1) / t.bn);
  const long slots = cus * t.blocks;
  const double per_round = (double)t.blocks * t.bm * t.bn / 65536.0 * (t.alpha * K / 1024.0 + t.eps[epi & 3]);
  return (double)((tiles + slots - 1) / slots) * per_round;
}

// How to cover an M x N output: one launch of `tile`, or (body_rows > 0) the first body_rows rows
// with `tile` and the rest with 128 x 128 tiles.  The second form cuts the output behind the last
// full round of the large tile, so that what would have been a partial round of whole-tile
// times becomes a round of small tiles: 32768 x 3200 in 256 x 256 tiles is 1664 tiles = 6.5
// rounds, priced 7; cut after 30208 rows it is 6 rounds plus 500 small tiles.
struct TilePlan { int tile, body_rows; double cost; };

static TilePlan plan_tiles(int M, int N, int K, int epi, bool may_split, long cus) {
  TilePlan best = {0, 0, tile_cost(M, N, K, epi, kShape256, cus)};
  const double keep = 0.98 * best.cost;          // the plain 256 x 256 launch stays unless clearly beaten
  auto offer = [&](int tile, int body_rows, double cost) {
    if (cost < keep && cost < best.cost) best = {tile, body_rows, cost};
  };
  offer(kShape128.cfg, 0, tile_cost(M, N, K, epi, kShape128, cus));
  offer(kShape320.cfg, 0, tile_cost(M, N, K, epi, kShape320, cus));
  if (may_split) {
    for (const TileShape* t : {&kShape256, &kShape320}) {
      const long tm = (M + t->bm - 1) / t->bm, tn = (N + t->bn - 1) / t->bn;
      const long full = tm * tn / cus;                       // complete rounds of the large tile
      if (full < 1 || (tm * tn) % cus == 0) continue;
      const long body_tm = std::min(full * cus / tn, (long)(M / t->bm));   // whole row tiles within them
      if (body_tm < 1 || body_tm * t->bm >= M) continue;
      const int body_rows = (int)body_tm * t->bm;
      offer(t->cfg, body_rows, tile_cost(body_rows, N, K, epi, *t, cus) + tile_cost(M - body_rows, N, K, epi, kShape128, cus) + kSecondLaunch);
    }
  }
  return best;
}

template <int EPI, int OUT, bool GATHER>
static void launch_epi(const GemmArgs& g, hipStream_t s) {
  int t = g.tile_cfg > 0 ? g.tile_cfg - 1 : -1;   // tile_cfg: set by the tuning hook of the C ABI, or by a split
  if (t != 0 && t != 2 && t != 4 && t != 5) t = plan_tiles(g.M, g.N, g.K, g.epilogue, false, g.compute_units > 0 ? g.compute_units : num_cus()).tile;
  if (EPI == EPI_QKV && (t == 0 || t == 5) && g.qk_cols % 256 != 0) t = 2;
  switch (t) {
    case 0: launch_cfg<T0, EPI, OUT, GATHER>(g, s); break;
    case 2: launch_cfg<T2, EPI, OUT, GATHER>(g, s); break;
    case 5: launch_cfg<T5, EPI, OUT, GATHER>(g, s); break;
    default: launch_cfg<T4, EPI, OUT, GATHER>(g, s); break;
  }
}

constexpr int kQkvBN = 128;

static void launch_gemm_bf16_whole(const GemmArgs& g, hipStream_t s);

// a forced tile, gathered rows, or Q | K columns that do not end on a 256-column boundary (those
// run the 256 x 128 tile): one launch
static bool may_split_rows(const GemmArgs& g) {
  return g.tile_cfg == 0 && !g.gather && !(g.epilogue == EPI_QKV && g.qk_cols % 256 != 0);
}

void plan_gemm_bf16(const GemmArgs& g, int compute_units, int* tile_rows, int* tile_cols, int* body_rows) {
  const long cus = compute_units > 0 ? compute_units : (g.compute_units > 0 ? g.compute_units : num_cus());
  int t = g.tile_cfg > 0 ? g.tile_cfg - 1 : -1, body = 0;
  if (t != 0 && t != 2 && t != 4 && t != 5) {
    const TilePlan p = plan_tiles(g.M, g.N, g.K, g.epilogue, may_split_rows(g), cus);
    t = p.tile; body = p.body_rows;
  }
  if (g.epilogue == EPI_QKV && (t == 0 || t == 5) && g.qk_cols % 256 != 0) t = 2;
  *tile_rows = t == 4 ? 128 : t == 5 ? 320 : 256;
  *tile_cols = t == 4 || t == 2 ? 128 : 256;
  *body_rows = body;
}

void launch_gemm_bf16(const GemmArgs& g, hipStream_t s) {
  if (g.M <= 0 || g.N <= 0) return;
  const TilePlan plan = may_split_rows(g) ? plan_tiles(g.M, g.N, g.K, g.epilogue, true, g.compute_units > 0 ? g.compute_units : num_cus()) : TilePlan{0, 0, 0.0};
  if (plan.body_rows <= 0) { launch_gemm_bf16_whole(g, s); return; }
  const int mb = plan.body_rows;
  GemmArgs body = g, tail = g;
  body.M = mb; body.tile_cfg = plan.tile + 1;
  tail.M = g.M - mb; tail.tile_cfg = kShape128.cfg + 1;
  // everything indexed by the output row moves down by mb rows (vt is indexed through vcol)
  tail.A = (const __bf16*)g.A + (size_t)mb * g.lda;
  if (g.out) tail.out = g.out_f32 ? (void*)((float*)g.out + (size_t)mb * g.ldo) : (void*)((__bf16*)g.out + (size_t)mb * g.ldo);
  if (g.resid) tail.resid = g.resid + (size_t)mb * g.ldr;
  if (g.xb) tail.xb = (__bf16*)g.xb + (size_t)mb * g.ldxb;
  if (g.stats_out) tail.stats_out = g.stats_out + (size_t)mb * g.stats_n;
  if (g.stats_in) tail.stats_in = g.stats_in + (size_t)mb * g.stats_n;
  if (g.rot) tail.rot = g.rot + (size_t)mb * g.rot_pairs;
  if (g.vcol) tail.vcol = g.vcol + mb;
  launch_gemm_bf16_whole(body, s);
  launch_gemm_bf16_whole(tail, s);
}

static void launch_gemm_bf16_whole(const GemmArgs& g, hipStream_t s) {
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
        v.W = (const __bf16*)g.W + (size_t)g.qk_cols * (g.ldw ? g.ldw : g.K);
        v.bias = g.bias ? (const void*)((const __bf16*)g.bias + g.qk_cols) : nullptr;
        v.N = g.N - g.qk_cols;
        v.qk_cols = 0;
        launch_epi<EPI_QKV, OUT_BF16, false>(v, s);
      }
      break;
  }
}

}  // namespace epd
