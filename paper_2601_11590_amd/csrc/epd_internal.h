// Internal declarations shared by the C-ABI layer and the kernel files of the Encode-stage
// library (V_m = E(I_m), paper section 3.1, Eq. 1).  Not installed; the public interface is
// include/epd_encode.h.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace epd {

// ---------------------------------------------------------------- GEMM description
// C[M,N] = A[M,K] * W[N,K]^T (+ bias[N]) followed by one of the epilogues below.
enum Epilogue : int {
  EPI_STORE = 0,     // out[m][n] = acc + bias               (out dtype: see out_f32)
  EPI_GELU = 1,      // out[m][n] = act(acc + bias)
  EPI_RESIDUAL = 2,  // resid[m][n] += acc + bias            (fp32 residual stream, in place)
  EPI_QKV = 3        // columns < qk_cols: rotate adjacent pairs by rot[m][.], store to out;
                     // columns >= qk_cols: V.  fp32 path stores V to out as well; the bf16
                     // path stores V transposed into vt[(n - qk_cols)][vcol[m]].
};

struct GemmArgs {
  const void* A;        // [M, K] row-major, leading dimension lda (elements)
  int lda;
  const int32_t* gather;  // optional [M, gather_n]: row m of A is the concatenation of rows
  int gather_n;           //   gather[m][0..gather_n) of A, each K/gather_n wide
  const void* W;        // [N, K] row-major, leading dimension ldw (elements; 0 = K)
  int ldw;
  const void* bias;     // [N] or nullptr
  int M, N, K;
  int epilogue;         // Epilogue
  int act;              // 0 = GELU erf, 1 = GELU tanh (EPI_GELU)
  void* out;            // [M, ldo]
  int ldo;
  int out_f32;          // bf16 path only: 1 = out is fp32 (patch embed writes the residual stream)
  float* resid;         // [M, ldr] (EPI_RESIDUAL)
  int ldr;
  // EPI_QKV
  const float2* rot;    // [M, rot_pairs] (cos, sin); nullptr = no rotary
  int rot_pairs;        // head_dim / 2
  int head_dim;
  int qk_cols;          // 2 * hidden
  float q_scale;        // bf16 path: columns < q_cols (the Q third) are multiplied by this after the
  int q_cols;           //   rotation, before rounding (0 = no scaling)
  void* vt;             // bf16 [hidden, vt_stride] transposed V
  int vt_stride;
  const int32_t* vcol;  // [M] column of token m in vt
  const void* zeros;    // bf16 path: >= 16 readable zero bytes (source of out-of-range tile chunks)
  int overread_ok;      // bf16 path: 1 = rows [M, round_up(M, 320)) of A and [N, round_up(N, 256)) of
                        //   W are readable memory (contents irrelevant): enables the load path
                        //   without per-lane row clamping
  // bf16 path, RMSNorm folded into the GEMMs around it (see launch_fold_gamma):
  //   producer (EPI_RESIDUAL): also store the updated residual rows as bf16 to xb and the sum
  //   of their squares per 128-column segment to stats_out[m][n / 128]
  void* xb;             // bf16 [M, ldxb] or nullptr
  int ldxb;
  float* stats_out;     // [M, stats_n] or nullptr (requires N % 128 == 0)
  //   consumer (any epilogue): the accumulator of row m is multiplied by
  //   rsqrt(sum_j stats_in[m][j] * stats_inv_dim + stats_eps) before bias / rotary / activation
  const float* stats_in;  // [M, stats_n] or nullptr
  int stats_n;
  float stats_inv_dim, stats_eps;
  int tile_cfg;         // bf16 path: 0 = automatic choice, k > 0 = tile variant k - 1 (tuning)
  int group_m;          // bf16 path: row tiles per rasterisation group (set by the launcher)
  int compute_units;    // bf16 path: compute units the launch will run on (a CU-masked stream); 0 = all of the device's
  int name_tag;         // bf16 path, EPI_RESIDUAL: 1 = the second MLP GEMM (a kernel name of its own in
                        //   profiles; the code is the same)
};

// ---------------------------------------------------------------- attention description
// One work item = one tile of query rows of one segment; the grid holds one block per
// (head, work item).
struct AttnWork { int32_t q0, seg_start, seg_len, vcol0; };

struct AttnArgs {
  const void* qkv;      // fp32 path: [T, 3D] (Q | K | V); bf16 path: [T, 2D] (Q | K)
  int ld_qkv;
  const void* vt;       // bf16 path: [D, vt_stride]
  int vt_stride;
  void* out;            // [T, D]
  int ld_out;
  const AttnWork* work;
  int num_work;
  int num_heads, head_dim;
  float scale;          // 1 / sqrt(head_dim); fp32 path only -- the bf16 path expects Q already
                        //   multiplied by scale * log2(e) (GemmArgs::q_scale)
  int q_tile;           // query rows per work item (attn_q_tile of this call: 128 or 256 on the bf16 path)
};

// ---------------------------------------------------------------- plan (per-call metadata)
struct PlanArgs {
  int T, Tm, num_items, num_segments;
  const int32_t* item_tok_off;  // device [items + 1]
  const int32_t* item_mrg_off;  // device [items + 1]
  const int32_t* grid_thw;      // device [items, 3]
  const int32_t* cu;            // device [segments + 1]
  const int32_t* pcu;           // device [segments + 1] padded segment starts in vt
  const double* pair_freq;      // device [pairs]
  const int32_t* pair_axis;     // device [pairs]
  int pairs;                    // 0 = no rotary
  int merge;
  float2* rot;                  // out [T, pairs]
  int32_t* merge_idx;           // out [Tm, merge*merge]
  int32_t* vcol;                // out [T] or nullptr
  void* vt;                     // bf16 [D, vt_stride]: pad columns are cleared, or nullptr
  int vt_stride, hidden;
};

// launchers (each checks nothing: shapes are validated by the caller); all asynchronous
void launch_plan(const PlanArgs& p, hipStream_t s);
void launch_norm(const float* x, const void* gamma, const void* beta, void* out, int T, int D,
                 float eps, bool rms, bool bf16, hipStream_t s);
void launch_gemm_f32(const GemmArgs& g, hipStream_t s);
bool launch_attn_f32(const AttnArgs& a, hipStream_t s);   // false: head_dim not covered
void launch_gemm_bf16(const GemmArgs& g, hipStream_t s);
// How launch_gemm_bf16 would tile g on a chip of compute_units units (<= 0: the current device's;
// host only, launches nothing): the tile of the first or only launch, and the rows that launch
// covers when the rest is left to a second launch of 128 x 128 tiles (0 = one launch covers all).
// Reads M, N, epilogue, qk_cols, gather and tile_cfg of g.
void plan_gemm_bf16(const GemmArgs& g, int compute_units, int* tile_rows, int* tile_cols, int* body_rows);
bool launch_attn_bf16(const AttnArgs& a, hipStream_t s);  // false: head_dim not covered
// query rows per work item for segments up to max_seg_len (0 = unsupported head_dim);
// never smaller than attn_q_tile(bf16, head_dim, 1).  groups: 0 = the library's choice; 1 or 2 =
// 128 or 256 query rows per work item on the bf16 path (256 = two 32-row groups per wave for
// head_dim <= 64, eight waves of one group above; 0 is returned where the request has no kernel)
int attn_q_tile(bool bf16, int head_dim, int max_seg_len, int groups = 0);
// W[n][k] *= gamma[k] (bf16, in place): folds the scale of an RMSNorm into the weights of the
// linear layer that consumes its output, so that  (x * rstd * gamma) W^T = rstd * (x (W gamma)^T)
void launch_fold_gamma(void* w, const void* gamma, int N, int K, hipStream_t s);
// dst[(sec, h, 2p+e)] = src[(sec, h, p + e*pairs)] for the Q and K sections, V copied
void launch_permute_qkv(const void* src_w, const void* src_b, void* dst_w, void* dst_b,
                        int hidden, int num_heads, int head_dim, int elem_bytes, hipStream_t s);

// ---------------------------------------------------------------- raw pixels -> patch rows
constexpr int kPrepItems = 32;      // items per launch (descriptors travel as kernel arguments)
constexpr int kPrepChannels = 8;
struct PrepItem {
  long long src_off;     // byte offset of the item's first pixel
  int hs, ws;            // source frame size
  int t, h, w;           // grid in patches
  int tok_off;           // first packed row of the item
  int blk_off;           // first token of the item in this launch (blockIdx.x counts tokens)
};
struct PrepArgs {
  const uint8_t* pixels;
  void* out;             // [T, pdim] bf16 or fp32
  int out_bf16;
  int n_items, channels, patch, tp, pdim;
  float a[kPrepChannels], b[kPrepChannels];    // value = pixel * a[c] + b[c]
  PrepItem item[kPrepItems];
};
void launch_preprocess(const PrepArgs& a, int tokens, hipStream_t s);   // patch <= 32 (block = patch/2 x patch)

constexpr int kVtAlign = 128;   // segment starts in the transposed-V buffer are multiples of this

}  // namespace epd
