// C-ABI layer of the Encode-stage library: V_m = E(I_m), V_m in R^{n x d} (paper section
// 3.1, Eq. 1).  Host-side only: validates, partitions the caller's workspace, builds the
// per-call plan (segment / item offsets, attention work list), and enqueues the kernels of
// the ViT forward pass on the caller's stream.  No device memory is allocated here.
#include "../../include/epd_encode.h"
#include "epd_internal.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

using namespace epd;

namespace {

thread_local std::string g_create_error = "";

constexpr size_t kAlign = 256;
constexpr int kStagingSlots = 4;
constexpr int kMaxTimedLaunches = 16384;

inline size_t align_up(size_t v, size_t a = kAlign) { return (v + a - 1) / a * a; }

std::string fmt(const char* f, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, f);
  vsnprintf(buf, sizeof(buf), f, ap);
  va_end(ap);
  return buf;
}

// ------------------------------------------------------------------ workspace layout
struct LayerW {   // byte offsets into the workspace; SIZE_MAX = absent
  size_t norm1_g, norm1_b, qkv_w, qkv_b, proj_w, proj_b, norm2_g, norm2_b, fc1_w, fc1_b, fc2_w, fc2_b;
};

struct Layout {
  int es;            // element size of cfg.dtype
  int pdim, pairs, mm, max_tm, max_work, vt_stride;
  int fpad;          // leading dimension of Hd and of the fc2 weights: mlp_dim, padded to 64 on the bf16 path
  size_t patch_w, patch_b, final_g, final_b, merge_w, merge_b;
  std::vector<LayerW> layers;
  size_t x, xn, qkv, vt, o, hd, rot, merge_idx, vcol, pair_freq, pair_axis, zeros, meta, stats;
  bool fold_rms;     // RMSNorm of the blocks folded into the GEMMs around it (bf16 path)
  int stats_n;       // 128-column segments per residual row
  size_t meta_bytes, total;
};

constexpr size_t kAbsent = (size_t)-1;

int q_tile(const epd_encode_cfg& c, int max_seg_len) { return attn_q_tile(c.dtype == EPD_BF16, c.head_dim, max_seg_len); }

Layout make_layout(const epd_encode_cfg& c) {
  Layout L;
  const bool bf = c.dtype == EPD_BF16;
  L.es = bf ? 2 : 4;
  const size_t es = L.es;
  const size_t D = c.hidden, F = c.mlp_dim, T = c.max_tokens;
  L.pdim = c.in_channels * c.temporal_patch * c.patch * c.patch;
  L.pairs = c.rope == EPD_ROPE_NONE ? 0 : c.head_dim / 2;
  L.mm = c.merge * c.merge;
  L.max_tm = c.max_tokens / L.mm;
  L.max_work = c.max_tokens / q_tile(c, 1) + c.max_segments + 1;   // smallest tile the kernels use
  // bf16: the K dimension of the fc2 GEMM is padded with zeros to a multiple of the K step, so
  // that it takes the GEMM's fast load path for any mlp_dim (4304 -> 4352)
  L.fpad = bf ? (int)align_up((size_t)c.mlp_dim, 64) : c.mlp_dim;
  L.vt_stride = (int)align_up((size_t)c.max_tokens + (size_t)c.max_segments * kVtAlign, kVtAlign);
  const bool ln = c.norm == EPD_LAYERNORM, bias = c.use_bias != 0;
  size_t off = 0;
  auto take = [&](size_t bytes, bool present = true) {
    if (!present) return kAbsent;
    size_t o = off;
    off = align_up(off + bytes);
    return o;
  };
  L.patch_w = take(D * L.pdim * es);
  L.patch_b = take(D * es, bias);
  L.final_g = take(D * es, c.final_norm != 0);
  L.final_b = take(D * es, c.final_norm != 0 && ln);
  L.merge_w = take((size_t)c.out_dim * L.mm * D * es);
  L.merge_b = take((size_t)c.out_dim * es, bias);
  L.layers.resize(c.num_layers);
  for (auto& w : L.layers) {
    w.norm1_g = take(D * es);
    w.norm1_b = take(D * es, ln);
    w.qkv_w = take(3 * D * D * es);
    w.qkv_b = take(3 * D * es, bias);
    w.proj_w = take(D * D * es);
    w.proj_b = take(D * es, bias);
    w.norm2_g = take(D * es);
    w.norm2_b = take(D * es, ln);
    w.fc1_w = take(F * D * es);
    w.fc1_b = take(F * es, bias);
    w.fc2_w = take(D * (size_t)L.fpad * es);
    w.fc2_b = take(D * es, bias);
  }
  L.x = take(T * D * 4);
  L.xn = take(T * D * es);
  L.qkv = take(T * (bf ? 2 : 3) * D * es);
  L.vt = take(D * (size_t)L.vt_stride * 2, bf);
  L.o = take(T * D * es);
  L.hd = take(T * (size_t)L.fpad * es);
  L.rot = take(T * (size_t)std::max(L.pairs, 1) * sizeof(float2));
  L.merge_idx = take((size_t)std::max(L.max_tm, 1) * L.mm * 4);
  L.vcol = take(T * 4, bf);
  L.pair_freq = take((size_t)std::max(L.pairs, 1) * 8);
  L.pair_axis = take((size_t)std::max(L.pairs, 1) * 4);
  L.zeros = take(256);
  const size_t S = c.max_segments, I = c.max_items;
  L.meta_bytes = align_up(((S + 1) * 2 + (I + 1) * 2 + 3 * I + 4 * (size_t)L.max_work) * 4);
  L.meta = take(L.meta_bytes);
  // bf16 + RMSNorm + hidden a multiple of 128: the block norms are not run as kernels.  The
  // residual GEMMs leave the raw rows in bf16 (in the Xn buffer) and their sums of squares per
  // 128-column segment; the consuming GEMM scales its accumulator rows by the resulting
  // 1/rms, gamma being folded into its weights at create.
  L.fold_rms = bf && c.norm == EPD_RMSNORM && c.hidden % 128 == 0 && c.num_layers > 0;
  L.stats_n = c.hidden / 128;
  L.stats = take(T * (size_t)std::max(L.stats_n, 1) * 4, L.fold_rms);
  // The bf16 GEMMs fetch whole operand tiles (up to 320 rows) without clamping rows at the edge of a
  // matrix (what lies beyond only feeds accumulators that are never stored); this tail keeps
  // such reads, from whichever buffer they start, inside the workspace.
  if (bf) take(320 * std::max(std::max(D, (size_t)L.fpad), (size_t)L.mm * D) * es);
  L.total = off;
  return L;
}

// ------------------------------------------------------------------ validation (host only)
epd_status validate_cfg(const epd_encode_cfg* c, bool need_buffers, std::string& err) {
  if (!c) { err = "cfg is NULL"; return EPD_ERR_INVALID_ARG; }
  if (c->struct_size != sizeof(epd_encode_cfg)) {
    err = fmt("cfg.struct_size %u != %zu", c->struct_size, sizeof(epd_encode_cfg));
    return EPD_ERR_INVALID_ARG;
  }
  if (c->dtype != EPD_F32 && c->dtype != EPD_BF16) { err = "cfg.dtype invalid"; return EPD_ERR_INVALID_ARG; }
  if (c->norm != EPD_LAYERNORM && c->norm != EPD_RMSNORM) { err = "cfg.norm invalid"; return EPD_ERR_INVALID_ARG; }
  if (c->act != EPD_GELU_ERF && c->act != EPD_GELU_TANH) { err = "cfg.act invalid"; return EPD_ERR_INVALID_ARG; }
  if (c->rope != EPD_ROPE_NONE && c->rope != EPD_ROPE_2D && c->rope != EPD_ROPE_3D) {
    err = "cfg.rope invalid"; return EPD_ERR_INVALID_ARG;
  }
  if (c->num_layers < 0 || c->hidden <= 0 || c->num_heads <= 0 || c->head_dim <= 0 || c->mlp_dim <= 0 ||
      c->in_channels <= 0 || c->patch <= 0 || c->temporal_patch <= 0 || c->merge <= 0 || c->out_dim <= 0 ||
      c->max_tokens <= 0 || c->max_segments <= 0 || c->max_items <= 0 || !(c->norm_eps >= 0.f)) {
    err = "cfg has a non-positive size field"; return EPD_ERR_INVALID_ARG;
  }
  if ((int64_t)c->num_heads * c->head_dim != c->hidden) {
    err = fmt("hidden %d != num_heads %d * head_dim %d", c->hidden, c->num_heads, c->head_dim);
    return EPD_ERR_UNSUPPORTED;
  }
  if (c->head_dim % 2) { err = "head_dim must be even"; return EPD_ERR_UNSUPPORTED; }
  if (c->rope != EPD_ROPE_NONE) {
    if (c->rope_pairs[0] < 0 || c->rope_pairs[1] < 0 || c->rope_pairs[2] < 0 ||
        c->rope_pairs[0] + c->rope_pairs[1] + c->rope_pairs[2] != c->head_dim / 2) {
      err = fmt("rope_pairs must be >= 0 and sum to head_dim/2 = %d", c->head_dim / 2);
      return EPD_ERR_UNSUPPORTED;
    }
    if (!(c->rope_base > 0.f)) { err = "rope_base must be positive"; return EPD_ERR_INVALID_ARG; }
  }
  if (c->merge > 8) { err = "merge > 8"; return EPD_ERR_UNSUPPORTED; }
  if (c->hidden > 8192) { err = "hidden > 8192"; return EPD_ERR_UNSUPPORTED; }
  const int pdim = c->in_channels * c->temporal_patch * c->patch * c->patch;
  if (c->dtype == EPD_BF16) {
    if (c->head_dim % 8 || c->hidden % 8 || c->mlp_dim % 8 || pdim % 8 || c->out_dim % 8) {
      err = "bf16: head_dim, hidden, mlp_dim, patch length and out_dim must be multiples of 8";
      return EPD_ERR_UNSUPPORTED;
    }
    if (!c->final_norm) {
      err = "bf16: the merger reads the normalised bf16 activations, final_norm must be 1";
      return EPD_ERR_UNSUPPORTED;
    }
  } else if (c->hidden % 4) {
    err = "fp32: hidden must be a multiple of 4"; return EPD_ERR_UNSUPPORTED;
  }
  if (attn_q_tile(c->dtype == EPD_BF16, c->head_dim, 1) <= 0) {
    err = fmt("head_dim %d has no attention kernel for this dtype", c->head_dim);
    return EPD_ERR_UNSUPPORTED;
  }
  if ((int64_t)c->max_tokens + (int64_t)c->max_segments * kVtAlign > (1ll << 30)) {
    err = "max_tokens too large"; return EPD_ERR_UNSUPPORTED;
  }
  // the bf16 attention kernel addresses the K rows of a segment with 32-bit byte offsets
  // (rows of 2 * hidden bf16 values)
  if (c->dtype == EPD_BF16 && (int64_t)c->max_tokens * c->hidden * 4 >= (1ll << 32)) {
    err = "max_tokens * hidden too large (bf16: must stay below 2^30)"; return EPD_ERR_UNSUPPORTED;
  }
  // ... and the rows of one head's transposed V tile the same way: head_dim rows of
  // (max_tokens + 128 * max_segments) bf16 columns each
  if (c->dtype == EPD_BF16 &&
      (int64_t)c->head_dim * ((int64_t)c->max_tokens + (int64_t)c->max_segments * kVtAlign + kVtAlign) * 2 >= (1ll << 32)) {
    err = "head_dim * (max_tokens + 128 * max_segments) too large (bf16: must stay below 2^31)";
    return EPD_ERR_UNSUPPORTED;
  }
  if (!need_buffers) return EPD_OK;
  const epd_weights* w = c->weights;
  if (!w) { err = "cfg.weights is NULL"; return EPD_ERR_INVALID_ARG; }
  const bool ln = c->norm == EPD_LAYERNORM, bias = c->use_bias != 0;
  bool ok = w->patch_w && w->merge_w && (!bias || (w->patch_b && w->merge_b)) &&
            (!c->final_norm || (w->final_norm_g && (!ln || w->final_norm_b))) &&
            (c->num_layers == 0 || w->layers);
  for (int l = 0; ok && l < c->num_layers; ++l) {
    const epd_layer_weights& lw = w->layers[l];
    ok = lw.norm1_g && lw.qkv_w && lw.proj_w && lw.norm2_g && lw.fc1_w && lw.fc2_w &&
         (!ln || (lw.norm1_b && lw.norm2_b)) && (!bias || (lw.qkv_b && lw.proj_b && lw.fc1_b && lw.fc2_b));
  }
  if (!ok) { err = "a required weight pointer is NULL"; return EPD_ERR_INVALID_ARG; }
  if (!c->workspace || ((uintptr_t)c->workspace % kAlign)) {
    err = "workspace is NULL or not 256-byte aligned"; return EPD_ERR_WORKSPACE;
  }
  return EPD_OK;
}

}  // namespace

// ------------------------------------------------------------------ handle
struct epd_encoder {
  epd_encode_cfg cfg;
  Layout L;
  char* ws = nullptr;
  std::string err;
  // pinned staging ring for per-call metadata
  char* staging = nullptr;
  hipEvent_t slot_done[kStagingSlots] = {};
  bool slot_used[kStagingSlots] = {};
  int next_slot = 0;
  int last_T = 0;
  // timing
  // tuning hook (epd_encode_set_tuning): 0 = the library's own choice
  int tile_cfg = 0;      // k > 0: bf16 GEMM tile variant k - 1
  int compute_units = 0; // > 0: the calls run on a stream masked to this many compute units
  int attn_groups = 0;   // 1 or 2: 128 or 256 query rows per block of the bf16 attention kernel
  int timed_step = -1;
  std::vector<hipEvent_t> ev;     // pairs (start, stop), created lazily
  int ev_used = 0;
  double timed_work = 0.0;

  template <typename P> P* at(size_t off) const { return off == kAbsent ? nullptr : (P*)(ws + off); }
};

namespace {

#define EPD_HIP(h, call)                                                                   \
  do {                                                                                     \
    hipError_t e_ = (call);                                                                \
    if (e_ != hipSuccess) {                                                                \
      (h)->err = fmt("%s failed: %s", #call, hipGetErrorString(e_));                       \
      return EPD_ERR_HIP;                                                                  \
    }                                                                                      \
  } while (0)

struct StepTimer {   // brackets one launch with events when its step is the timed one
  epd_encoder* h;
  hipStream_t s;
  bool on;
  StepTimer(epd_encoder* h_, int step, double work, hipStream_t s_) : h(h_), s(s_) {
    on = h->timed_step == step && h->ev_used + 2 <= kMaxTimedLaunches * 2;
    if (!on) return;
    while ((int)h->ev.size() < h->ev_used + 2) {
      hipEvent_t e;
      if (hipEventCreate(&e) != hipSuccess) { on = false; return; }
      h->ev.push_back(e);
    }
    h->timed_work += work;
    hipEventRecord(h->ev[h->ev_used], s);
  }
  ~StepTimer() {
    if (!on) return;
    hipEventRecord(h->ev[h->ev_used + 1], s);
    h->ev_used += 2;
  }
};

epd_status copy_weight(epd_encoder* h, size_t dst_off, const void* src, size_t bytes) {
  if (dst_off == kAbsent || !src) return EPD_OK;
  EPD_HIP(h, hipMemcpyAsync(h->ws + dst_off, src, bytes, hipMemcpyDeviceToDevice, 0));
  return EPD_OK;
}

}  // namespace

extern "C" {

uint64_t epd_encode_workspace_bytes(const epd_encode_cfg* cfg) {
  std::string err;
  if (validate_cfg(cfg, false, err) != EPD_OK) return 0;
  return make_layout(*cfg).total;
}

epd_status epd_encode_create(const epd_encode_cfg* cfg, epd_handle* out) {
  if (!out) { g_create_error = "out is NULL"; return EPD_ERR_INVALID_ARG; }
  epd_status st = validate_cfg(cfg, true, g_create_error);
  if (st != EPD_OK) return st;
  epd_encoder* h = new epd_encoder();
  h->cfg = *cfg;
  h->cfg.weights = nullptr;   // the caller's table is not kept
  h->L = make_layout(*cfg);
  h->ws = (char*)cfg->workspace;
  if (cfg->workspace_bytes < h->L.total) {
    g_create_error = fmt("workspace_bytes %llu < required %zu", (unsigned long long)cfg->workspace_bytes, h->L.total);
    delete h;
    return EPD_ERR_WORKSPACE;
  }
  auto fail = [&](epd_status s) {
    g_create_error = h->err;
    if (h->staging) (void)hipHostFree(h->staging);
    for (auto& e : h->slot_done) if (e) (void)hipEventDestroy(e);
    delete h;
    return s;
  };
  const Layout& L = h->L;
  const epd_weights& w = *cfg->weights;
  const size_t es = L.es, D = cfg->hidden, F = cfg->mlp_dim;
#define EPD_CW(dst, src, bytes)                                         \
  do {                                                                  \
    epd_status s_ = copy_weight(h, dst, src, bytes);                    \
    if (s_ != EPD_OK) return fail(s_);                                  \
  } while (0)
  EPD_CW(L.patch_w, w.patch_w, D * L.pdim * es);
  EPD_CW(L.patch_b, w.patch_b, D * es);
  EPD_CW(L.final_g, w.final_norm_g, D * es);
  EPD_CW(L.final_b, w.final_norm_b, D * es);
  EPD_CW(L.merge_w, w.merge_w, (size_t)cfg->out_dim * L.mm * D * es);
  EPD_CW(L.merge_b, w.merge_b, (size_t)cfg->out_dim * es);
  for (int l = 0; l < cfg->num_layers; ++l) {
    const epd_layer_weights& s = w.layers[l];
    const LayerW& d = L.layers[l];
    EPD_CW(d.norm1_g, s.norm1_g, D * es);
    EPD_CW(d.norm1_b, s.norm1_b, D * es);
    launch_permute_qkv(s.qkv_w, cfg->use_bias ? s.qkv_b : nullptr, h->ws + d.qkv_w,
                       d.qkv_b == kAbsent ? nullptr : h->ws + d.qkv_b, cfg->hidden, cfg->num_heads,
                       cfg->head_dim, L.es, 0);
    EPD_CW(d.proj_w, s.proj_w, D * D * es);
    EPD_CW(d.proj_b, s.proj_b, D * es);
    EPD_CW(d.norm2_g, s.norm2_g, D * es);
    EPD_CW(d.norm2_b, s.norm2_b, D * es);
    EPD_CW(d.fc1_w, s.fc1_w, F * D * es);
    EPD_CW(d.fc1_b, s.fc1_b, F * es);
    if (L.fpad == (int)F) {
      EPD_CW(d.fc2_w, s.fc2_w, D * F * es);
    } else {   // rows of mlp_dim elements into rows of fpad, the pad cleared
      if (!s.fc2_w) return fail(EPD_ERR_INVALID_ARG);
      if (hipMemsetAsync(h->ws + d.fc2_w, 0, D * (size_t)L.fpad * es, 0) != hipSuccess ||
          hipMemcpy2DAsync(h->ws + d.fc2_w, (size_t)L.fpad * es, s.fc2_w, F * es, F * es, D, hipMemcpyDeviceToDevice, 0) != hipSuccess) {
        h->err = "copying the fc2 weights failed";
        return fail(EPD_ERR_HIP);
      }
    }
    EPD_CW(d.fc2_b, s.fc2_b, D * es);
    if (L.fold_rms) {
      // norm2 -> fc1 in every block; norm1 -> qkv from the second block on (the first block's
      // norm1 follows the patch embedding and runs as a kernel)
      launch_fold_gamma(h->ws + d.fc1_w, h->ws + d.norm2_g, (int)F, (int)D, 0);
      if (l > 0) launch_fold_gamma(h->ws + d.qkv_w, h->ws + d.norm1_g, 3 * (int)D, (int)D, 0);
    }
  }
#undef EPD_CW
  // rotary frequencies per pair (double) and the axis each pair belongs to
  if (L.pairs > 0) {
    std::vector<double> freq(L.pairs);
    std::vector<int32_t> axis(L.pairs);
    int p = 0;
    for (int a = 0; a < 3; ++a)
      for (int j = 0; j < cfg->rope_pairs[a]; ++j, ++p) {
        freq[p] = std::pow((double)cfg->rope_base, -(double)j / (double)cfg->rope_pairs[a]);
        axis[p] = a;
      }
    hipError_t e = hipMemcpy(h->ws + L.pair_freq, freq.data(), L.pairs * 8, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(h->ws + L.pair_axis, axis.data(), L.pairs * 4, hipMemcpyHostToDevice);
    if (e != hipSuccess) { h->err = fmt("rotary table upload failed: %s", hipGetErrorString(e)); return fail(EPD_ERR_HIP); }
  }
  if (L.fpad != cfg->mlp_dim) {   // pad columns of Hd stay zero: the fc1 GEMM never writes them
    hipError_t e0 = hipMemsetAsync(h->ws + L.hd, 0, (size_t)cfg->max_tokens * L.fpad * es, 0);
    if (e0 != hipSuccess) { h->err = fmt("hipMemsetAsync failed: %s", hipGetErrorString(e0)); return fail(EPD_ERR_HIP); }
  }
  hipError_t e = hipMemsetAsync(h->ws + L.zeros, 0, 256, 0);
  if (e != hipSuccess) { h->err = fmt("hipMemsetAsync failed: %s", hipGetErrorString(e)); return fail(EPD_ERR_HIP); }
  e = hipHostMalloc((void**)&h->staging, L.meta_bytes * kStagingSlots, hipHostMallocDefault);
  if (e != hipSuccess) { h->staging = nullptr; h->err = fmt("hipHostMalloc failed: %s", hipGetErrorString(e)); return fail(EPD_ERR_HIP); }
  for (auto& ev : h->slot_done) {
    e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
    if (e != hipSuccess) { ev = nullptr; h->err = fmt("hipEventCreate failed: %s", hipGetErrorString(e)); return fail(EPD_ERR_HIP); }
  }
  e = hipStreamSynchronize(0);
  if (e == hipSuccess) e = hipGetLastError();
  if (e != hipSuccess) { h->err = fmt("weight copy failed: %s", hipGetErrorString(e)); return fail(EPD_ERR_HIP); }
  *out = h;
  return EPD_OK;
}

epd_status epd_encode(epd_handle h, const void* packed_patches, const int32_t* cu_seqlens,
                      int32_t num_segments, const int32_t* grid_thw, int32_t num_items,
                      void* out_visual_tokens, void* stream) {
  if (!h) { g_create_error = "handle is NULL"; return EPD_ERR_INVALID_ARG; }
  if (!packed_patches || !cu_seqlens || !grid_thw || !out_visual_tokens) {
    h->err = "a required pointer is NULL"; return EPD_ERR_INVALID_ARG;
  }
  const epd_encode_cfg& c = h->cfg;
  const Layout& L = h->L;
  // ---- metadata checks: nothing is launched unless all of them hold
  if (num_segments <= 0 || num_segments > c.max_segments || num_items <= 0 || num_items > c.max_items) {
    h->err = fmt("num_segments %d (max %d) / num_items %d (max %d) out of range", num_segments, c.max_segments,
                 num_items, c.max_items);
    return EPD_ERR_SHAPE;
  }
  int64_t T64 = 0, Tm64 = 0;
  for (int i = 0; i < num_items; ++i) {
    int64_t t = grid_thw[3 * i], hh = grid_thw[3 * i + 1], ww = grid_thw[3 * i + 2];
    if (t <= 0 || hh <= 0 || ww <= 0 || hh % c.merge || ww % c.merge) {
      h->err = fmt("grid_thw[%d] = (%lld, %lld, %lld): sizes must be positive and h, w divisible by merge %d", i,
                   (long long)t, (long long)hh, (long long)ww, c.merge);
      return EPD_ERR_SHAPE;
    }
    T64 += t * hh * ww;
    Tm64 += t * (hh / c.merge) * (ww / c.merge);
    if (T64 > c.max_tokens) { h->err = fmt("more than max_tokens = %d tokens", c.max_tokens); return EPD_ERR_SHAPE; }
  }
  if (cu_seqlens[0] != 0 || cu_seqlens[num_segments] != T64) {
    h->err = fmt("cu_seqlens must run from 0 to T = %lld", (long long)T64); return EPD_ERR_SHAPE;
  }
  for (int s = 0; s < num_segments; ++s)
    if (cu_seqlens[s + 1] <= cu_seqlens[s]) { h->err = fmt("cu_seqlens not strictly increasing at %d", s); return EPD_ERR_SHAPE; }
  const int T = (int)T64, Tm = (int)Tm64;
  const bool bf = c.dtype == EPD_BF16;
  hipStream_t st = (hipStream_t)stream;

  // ---- per-call metadata -> pinned staging slot -> device
  const int slot = h->next_slot;
  if (h->slot_used[slot]) EPD_HIP(h, hipEventSynchronize(h->slot_done[slot]));
  int32_t* m = (int32_t*)(h->staging + (size_t)slot * L.meta_bytes);
  const int S = num_segments, I = num_items;
  int32_t* cu = m;
  int32_t* pcu = cu + (S + 1);
  int32_t* ioff = pcu + (S + 1);
  int32_t* moff = ioff + (I + 1);
  int32_t* grid = moff + (I + 1);
  AttnWork* work = (AttnWork*)(grid + 3 * I);
  std::memcpy(cu, cu_seqlens, (S + 1) * 4);
  pcu[0] = 0;
  for (int s = 0; s < S; ++s) pcu[s + 1] = (int32_t)align_up((size_t)pcu[s] + (cu[s + 1] - cu[s]), kVtAlign);
  ioff[0] = moff[0] = 0;
  for (int i = 0; i < I; ++i) {
    int t = grid_thw[3 * i], hh = grid_thw[3 * i + 1], ww = grid_thw[3 * i + 2];
    ioff[i + 1] = ioff[i] + t * hh * ww;
    moff[i + 1] = moff[i] + t * (hh / c.merge) * (ww / c.merge);
    grid[3 * i] = t; grid[3 * i + 1] = hh; grid[3 * i + 2] = ww;
  }
  // attention work list: one entry per query tile, longest segments first so that the tail
  // of the launch is made of short items
  int max_len = 0;
  for (int s = 0; s < S; ++s) max_len = std::max(max_len, cu[s + 1] - cu[s]);
  const int bq = attn_q_tile(bf, c.head_dim, max_len, h->attn_groups);
  if (bq <= 0) { h->err = "internal: no attention kernel for the forced query tile"; return EPD_ERR_UNSUPPORTED; }
  std::vector<int> order(S);
  for (int s = 0; s < S; ++s) order[s] = s;
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return cu[a + 1] - cu[a] > cu[b + 1] - cu[b]; });
  int nwork = 0;
  for (int s : order) {
    const int len = cu[s + 1] - cu[s];
    for (int q0 = 0; q0 < len; q0 += bq) work[nwork++] = AttnWork{cu[s] + q0, cu[s], len, pcu[s]};
  }
  if (nwork > L.max_work) { h->err = "internal: attention work list overflow"; return EPD_ERR_SHAPE; }
  const size_t meta_used = (size_t)((char*)(work + nwork) - (char*)m);
  EPD_HIP(h, hipMemcpyAsync(h->ws + L.meta, m, meta_used, hipMemcpyHostToDevice, st));
  EPD_HIP(h, hipEventRecord(h->slot_done[slot], st));
  h->slot_used[slot] = true;
  h->next_slot = (slot + 1) % kStagingSlots;

  const int32_t* d_cu = h->at<int32_t>(L.meta);
  const int32_t* d_pcu = d_cu + (S + 1);
  const int32_t* d_ioff = d_pcu + (S + 1);
  const int32_t* d_moff = d_ioff + (I + 1);
  const int32_t* d_grid = d_moff + (I + 1);
  const AttnWork* d_work = (const AttnWork*)(d_grid + 3 * I);

  const int D = c.hidden, F = c.mlp_dim;
  float* X = h->at<float>(L.x);
  void* Xn = h->at<void>(L.xn);
  void* QKV = h->at<void>(L.qkv);
  void* Vt = h->at<void>(L.vt);
  void* O = h->at<void>(L.o);
  void* Hd = h->at<void>(L.hd);
  float2* rot = L.pairs > 0 ? h->at<float2>(L.rot) : nullptr;
  int32_t* vcol = h->at<int32_t>(L.vcol);
  int32_t* midx = h->at<int32_t>(L.merge_idx);

  {
    StepTimer tm(h, EPD_STEP_PLAN, 0.0, st);
    PlanArgs p{};
    p.T = T; p.Tm = Tm; p.num_items = I; p.num_segments = S;
    p.item_tok_off = d_ioff; p.item_mrg_off = d_moff; p.grid_thw = d_grid; p.cu = d_cu; p.pcu = d_pcu;
    p.pair_freq = h->at<double>(L.pair_freq); p.pair_axis = h->at<int32_t>(L.pair_axis);
    p.pairs = L.pairs; p.merge = c.merge; p.rot = rot; p.merge_idx = midx;
    p.vcol = bf ? vcol : nullptr; p.vt = bf ? Vt : nullptr; p.vt_stride = L.vt_stride; p.hidden = D;
    launch_plan(p, st);
  }

  auto gemm = [&](int step, GemmArgs& g, int k_counted = 0) {   // k_counted: K without padding
    StepTimer tm(h, step, 2.0 * g.M * (double)g.N * (k_counted ? k_counted : g.K), st);
    g.zeros = h->ws + L.zeros;
    // operands that live in the workspace may be read past their last row (see make_layout)
    g.overread_ok = (g.A != packed_patches && !g.gather) ? 1 : 0;
    g.tile_cfg = h->tile_cfg;
    g.compute_units = h->compute_units;
    if (bf) launch_gemm_bf16(g, st); else launch_gemm_f32(g, st);
  };
  auto norm = [&](const void* gma, const void* bta, void* dst) {
    StepTimer tm(h, EPD_STEP_NORM, (double)T * D * (4.0 + L.es), st);
    launch_norm(X, gma, bta, dst, T, D, c.norm_eps, c.norm == EPD_RMSNORM, bf, st);
  };

  {  // patch embedding: X = P Wpe^T + b   (fp32 residual stream)
    GemmArgs g{};
    g.A = packed_patches; g.lda = L.pdim; g.W = h->at<void>(L.patch_w); g.bias = h->at<void>(L.patch_b);
    g.M = T; g.N = D; g.K = L.pdim; g.epilogue = EPI_STORE; g.out = X; g.ldo = D; g.out_f32 = 1;
    gemm(EPD_STEP_PATCH_EMBED, g);
  }
  float* stats = L.fold_rms ? h->at<float>(L.stats) : nullptr;
  auto consume_stats = [&](GemmArgs& g) {   // A = raw bf16 rows, scale 1/rms applied in the epilogue
    g.stats_in = stats; g.stats_n = L.stats_n; g.stats_inv_dim = 1.0f / (float)D; g.stats_eps = c.norm_eps;
  };
  auto produce_stats = [&](GemmArgs& g) {   // residual GEMM also leaves bf16 rows + sums of squares
    g.xb = Xn; g.ldxb = D; g.stats_out = stats; g.stats_n = L.stats_n;
  };
  for (int l = 0; l < c.num_layers; ++l) {
    const LayerW& w = L.layers[l];
    const bool fold1 = L.fold_rms && l > 0;
    if (!fold1) norm(h->at<void>(w.norm1_g), h->at<void>(w.norm1_b), Xn);
    {  // QKV projection, rotary on Q and K in the epilogue
      GemmArgs g{};
      if (fold1) consume_stats(g);
      g.A = Xn; g.lda = D; g.W = h->at<void>(w.qkv_w); g.bias = h->at<void>(w.qkv_b);
      g.M = T; g.N = 3 * D; g.K = D; g.epilogue = EPI_QKV; g.out = QKV; g.ldo = bf ? 2 * D : 3 * D;
      g.rot = rot; g.rot_pairs = L.pairs; g.head_dim = c.head_dim; g.qk_cols = 2 * D;
      g.vt = Vt; g.vt_stride = L.vt_stride; g.vcol = vcol;
      if (bf) { g.q_cols = D; g.q_scale = (float)(1.4426950408889634 / std::sqrt((double)c.head_dim)); }
      gemm(EPD_STEP_QKV, g);
    }
    {  // block-diagonal non-causal attention
      AttnArgs a{};
      a.qkv = QKV; a.ld_qkv = bf ? 2 * D : 3 * D; a.vt = Vt; a.vt_stride = L.vt_stride;
      a.out = O; a.ld_out = D; a.work = d_work; a.num_work = nwork;
      a.num_heads = c.num_heads; a.head_dim = c.head_dim; a.q_tile = bq; a.scale = (float)(1.0 / std::sqrt((double)c.head_dim));
      double flops = 0.0;
      for (int s = 0; s < S; ++s) { double n = cu[s + 1] - cu[s]; flops += 4.0 * n * n * D; }
      StepTimer tm(h, EPD_STEP_ATTN, flops, st);
      bool ok = bf ? launch_attn_bf16(a, st) : launch_attn_f32(a, st);
      if (!ok) { h->err = "internal: no attention kernel"; return EPD_ERR_UNSUPPORTED; }
    }
    {  // X += O Wo^T + bo
      GemmArgs g{};
      g.A = O; g.lda = D; g.W = h->at<void>(w.proj_w); g.bias = h->at<void>(w.proj_b);
      g.M = T; g.N = D; g.K = D; g.epilogue = EPI_RESIDUAL; g.resid = X; g.ldr = D;
      if (L.fold_rms) produce_stats(g);
      gemm(EPD_STEP_PROJ, g);
    }
    if (!L.fold_rms) norm(h->at<void>(w.norm2_g), h->at<void>(w.norm2_b), Xn);
    {  // Hd = GELU(Xn W1^T + b1)
      GemmArgs g{};
      if (L.fold_rms) consume_stats(g);
      g.A = Xn; g.lda = D; g.W = h->at<void>(w.fc1_w); g.bias = h->at<void>(w.fc1_b);
      g.M = T; g.N = F; g.K = D; g.epilogue = EPI_GELU; g.act = c.act; g.out = Hd; g.ldo = L.fpad;
      gemm(EPD_STEP_FC1, g);
    }
    {  // X += Hd W2^T + b2
      GemmArgs g{};
      g.A = Hd; g.lda = L.fpad; g.W = h->at<void>(w.fc2_w); g.ldw = L.fpad; g.bias = h->at<void>(w.fc2_b);
      g.M = T; g.N = D; g.K = L.fpad;   // pad columns of Hd and of the weights are zero
      g.epilogue = EPI_RESIDUAL; g.resid = X; g.ldr = D;
      if (L.fold_rms && l + 1 < c.num_layers) produce_stats(g);
      g.name_tag = 1;
      gemm(EPD_STEP_FC2, g, (int)F);
    }
  }
  const void* Z = X;   // fp32 path without a final norm reads the residual stream directly
  if (c.final_norm) {
    norm(h->at<void>(L.final_g), h->at<void>(L.final_b), Xn);
    Z = Xn;
  }
  {  // merger: gather merge x merge neighbours, project
    GemmArgs g{};
    g.A = Z; g.lda = D; g.W = h->at<void>(L.merge_w); g.bias = h->at<void>(L.merge_b);
    g.M = Tm; g.N = c.out_dim; g.K = L.mm * D; g.epilogue = EPI_STORE; g.out = out_visual_tokens; g.ldo = c.out_dim;
    if (c.merge > 1) { g.gather = midx; g.gather_n = L.mm; }
    gemm(EPD_STEP_MERGE, g);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { h->err = fmt("kernel launch failed: %s", hipGetErrorString(e)); return EPD_ERR_HIP; }
  h->last_T = T;
  return EPD_OK;
}

epd_status epd_encode_destroy(epd_handle h) {
  if (!h) return EPD_ERR_INVALID_ARG;
  for (auto& e : h->slot_done) if (e) (void)hipEventDestroy(e);
  for (auto& e : h->ev) (void)hipEventDestroy(e);
  if (h->staging) (void)hipHostFree(h->staging);
  delete h;
  return EPD_OK;
}

const char* epd_encode_last_error(epd_handle h) { return h ? h->err.c_str() : g_create_error.c_str(); }

epd_status epd_encode_debug_hidden(epd_handle h, void* out_T_by_D_f32, void* stream) {
  if (!h || !out_T_by_D_f32) return EPD_ERR_INVALID_ARG;
  if (h->last_T <= 0) { h->err = "no completed epd_encode call"; return EPD_ERR_INVALID_ARG; }
  EPD_HIP(h, hipMemcpyAsync(out_T_by_D_f32, h->ws + h->L.x, (size_t)h->last_T * h->cfg.hidden * 4,
                            hipMemcpyDeviceToDevice, (hipStream_t)stream));
  return EPD_OK;
}

// Checks shared by the entry points that take raw pixels: everything that decides how far a
// kernel reads or writes is validated here, on the host, before anything is launched.
static epd_status check_raw_items(epd_handle h, const int32_t* src_hw, const int32_t* grid_thw, int32_t num_items,
                                  const float* mean, const float* stdv, bool for_encode) {
  const epd_encode_cfg& c = h->cfg;
  if (c.in_channels > kPrepChannels || c.patch % 2 || c.patch > 32 || c.in_channels * c.temporal_patch > 65535) {
    h->err = fmt("raw-pixel input covers up to %d channels and even patch sizes up to 32 (have %d, %d)", kPrepChannels,
                 c.in_channels, c.patch);
    return EPD_ERR_UNSUPPORTED;
  }
  if (num_items <= 0 || num_items > c.max_items) {
    h->err = fmt("num_items %d (max %d) out of range", num_items, c.max_items); return EPD_ERR_SHAPE;
  }
  constexpr int kMaxSide = 16384;     // keeps the tap arithmetic, (2j + 1) * n_in, inside 32 bits
  for (int ch = 0; ch < c.in_channels; ++ch)
    if (!(stdv[ch] > 0.f) || !std::isfinite(stdv[ch]) || !std::isfinite(mean[ch])) {
      h->err = fmt("mean / std of channel %d must be finite, std positive", ch); return EPD_ERR_INVALID_ARG;
    }
  int64_t T64 = 0;
  for (int i = 0; i < num_items; ++i) {
    const int64_t t = grid_thw[3 * i], hh = grid_thw[3 * i + 1], ww = grid_thw[3 * i + 2];
    const int64_t hs = src_hw[2 * i], ws = src_hw[2 * i + 1];
    if (t <= 0 || hh <= 0 || ww <= 0 || hs <= 0 || ws <= 0 || hs > kMaxSide || ws > kMaxSide ||
        hh * c.patch > kMaxSide || ww * c.patch > kMaxSide) {
      h->err = fmt("item %d: grid (%lld, %lld, %lld) / source size (%lld, %lld) must be positive, sides at most %d pixels",
                   i, (long long)t, (long long)hh, (long long)ww, (long long)hs, (long long)ws, kMaxSide);
      return EPD_ERR_SHAPE;
    }
    if (for_encode && (hh % c.merge || ww % c.merge)) {
      h->err = fmt("item %d: h, w must be divisible by merge %d", i, c.merge); return EPD_ERR_SHAPE;
    }
    T64 += t * hh * ww;
    if (T64 > c.max_tokens) { h->err = fmt("more than max_tokens = %d tokens", c.max_tokens); return EPD_ERR_SHAPE; }
  }
  if (for_encode && num_items > c.max_segments) {
    h->err = fmt("one attention segment per item: %d items exceed max_segments = %d", num_items, c.max_segments);
    return EPD_ERR_SHAPE;
  }
  return EPD_OK;
}

// Raw pixels -> packed patch rows (the step in front of epd_encode).  All checks are made on
// the host before anything is launched; item descriptors travel as kernel arguments,
// kPrepItems per launch, so the call touches neither the workspace nor the staging buffers.
epd_status epd_preprocess(epd_handle h, const uint8_t* pixels, const int32_t* src_hw, const int32_t* grid_thw,
                          int32_t num_items, const float* mean, const float* stdv, void* packed_patches,
                          void* stream) {
  if (!h) { g_create_error = "handle is NULL"; return EPD_ERR_INVALID_ARG; }
  if (!pixels || !src_hw || !grid_thw || !mean || !stdv || !packed_patches) {
    h->err = "a required pointer is NULL"; return EPD_ERR_INVALID_ARG;
  }
  const epd_encode_cfg& c = h->cfg;
  if (epd_status st = check_raw_items(h, src_hw, grid_thw, num_items, mean, stdv, false)) return st;
  PrepArgs a{};
  a.pixels = pixels; a.out = packed_patches; a.out_bf16 = c.dtype == EPD_BF16;
  a.channels = c.in_channels; a.patch = c.patch; a.tp = c.temporal_patch; a.pdim = h->L.pdim;
  for (int ch = 0; ch < c.in_channels; ++ch) {
    a.a[ch] = (float)(1.0 / (255.0 * (double)stdv[ch]));
    a.b[ch] = (float)(-(double)mean[ch] / (double)stdv[ch]);
  }
  long long src_off = 0;
  int tok_off = 0;
  for (int i0 = 0; i0 < num_items; i0 += kPrepItems) {
    const int n = std::min(kPrepItems, num_items - i0);
    long long blocks = 0;
    for (int j = 0; j < n; ++j) {
      const int i = i0 + j;
      PrepItem& d = a.item[j];
      d.t = grid_thw[3 * i]; d.h = grid_thw[3 * i + 1]; d.w = grid_thw[3 * i + 2];
      d.hs = src_hw[2 * i]; d.ws = src_hw[2 * i + 1];
      d.src_off = src_off; d.tok_off = tok_off; d.blk_off = (int)blocks;
      const long long tokens = (long long)d.t * d.h * d.w;
      blocks += tokens;
      src_off += (long long)c.in_channels * d.t * c.temporal_patch * d.hs * d.ws;
      tok_off += (int)tokens;
    }
    if (blocks > 0x7fffffffLL) { h->err = "internal: preprocess grid too large"; return EPD_ERR_SHAPE; }
    a.n_items = n;
    launch_preprocess(a, (int)blocks, (hipStream_t)stream);
  }
  EPD_HIP(h, hipGetLastError());
  return EPD_OK;
}

// Encode through the store (see the header): hash -> lookup -> copy the hits, preprocess and
// encode the misses as one compact batch, file them, copy them out.  Everything after the
// keys have arrived is asynchronous on one stream, so a pool range that an insert of this
// call recycles is overwritten only after the copies that still read it.
epd_status epd_encode_cached(epd_handle h, epd_store_handle s, uint64_t model_salt, const uint8_t* pixels,
                             const int32_t* src_hw, const int32_t* grid_thw, int32_t num_items, const float* mean,
                             const float* stdv, void* rows_scratch, void* out_scratch, void* out_visual_tokens,
                             int32_t* hit_out, uint64_t* keys_out, void* stream) {
  if (!h) { g_create_error = "handle is NULL"; return EPD_ERR_INVALID_ARG; }
  if (!s || !pixels || !src_hw || !grid_thw || !mean || !stdv || !rows_scratch || !out_scratch || !out_visual_tokens) {
    h->err = "a required pointer is NULL"; return EPD_ERR_INVALID_ARG;
  }
  if (epd_status st = check_raw_items(h, src_hw, grid_thw, num_items, mean, stdv, true)) return st;
  const epd_encode_cfg& c = h->cfg;
  hipStream_t st = (hipStream_t)stream;
  const size_t es = h->L.es, row_bytes = (size_t)c.out_dim * es;
  const int n = num_items;
  std::vector<uint64_t> off(n + 1, 0), salt(n), keys((size_t)n * 2);
  std::vector<int64_t> tok(n + 1, 0), mrg(n + 1, 0);
  for (int i = 0; i < n; ++i) {
    const int64_t t = grid_thw[3 * i], hh = grid_thw[3 * i + 1], ww = grid_thw[3 * i + 2];
    const int64_t hs = src_hw[2 * i], ws = src_hw[2 * i + 1];
    off[i + 1] = off[i] + (uint64_t)(c.in_channels * t * c.temporal_patch * hs * ws);
    tok[i + 1] = tok[i] + t * hh * ww;
    mrg[i + 1] = mrg[i] + t * (hh / c.merge) * (ww / c.merge);
    uint64_t x = model_salt;
    const int64_t f[9] = {hs, ws, t, hh, ww, c.patch, c.temporal_patch, c.in_channels, (int64_t)c.dtype};
    for (int64_t v : f) x = (x ^ (uint64_t)v) * 0x9E3779B97F4A7C15ull;
    salt[i] = x;
  }
  if (epd_status e = epd_store_hash(s, pixels, off.data(), salt.data(), n, keys.data(), stream)) {
    h->err = std::string("epd_store_hash: ") + epd_store_last_error(s); return e;
  }
  if (keys_out) std::memcpy(keys_out, keys.data(), keys.size() * 8);
  // hits: copy out; misses: collect
  std::vector<int> miss;
  for (int i = 0; i < n; ++i) {
    void* p = nullptr;
    uint64_t bytes = 0;
    const size_t want = (size_t)(mrg[i + 1] - mrg[i]) * row_bytes;
    const epd_status e = epd_store_lookup(s, &keys[2 * i], &p, &bytes);
    const bool hit = e == EPD_OK && bytes == want;
    if (hit_out) hit_out[i] = hit ? 1 : 0;
    if (hit) EPD_HIP(h, hipMemcpyAsync((char*)out_visual_tokens + (size_t)mrg[i] * row_bytes, p, want, hipMemcpyDeviceToDevice, st));
    else miss.push_back(i);
  }
  if (miss.empty()) return EPD_OK;
  // misses: preprocess every run of neighbouring items into the compact batch, then encode it
  std::vector<int32_t> cu(miss.size() + 1, 0), grid(miss.size() * 3);
  const size_t prow = (size_t)h->L.pdim * es;
  for (size_t k = 0; k < miss.size();) {
    size_t e = k + 1;
    while (e < miss.size() && miss[e] == miss[e - 1] + 1) ++e;
    const int i0 = miss[k], cnt = (int)(e - k);
    if (epd_status stt = epd_preprocess(h, pixels + off[i0], src_hw + 2 * i0, grid_thw + 3 * i0, cnt, mean, stdv,
                                        (char*)rows_scratch + (size_t)cu[k] * prow, stream)) return stt;
    for (size_t j = k; j < e; ++j) {
      const int i = miss[j];
      cu[j + 1] = cu[j] + (int32_t)(tok[i + 1] - tok[i]);
      grid[3 * j] = grid_thw[3 * i]; grid[3 * j + 1] = grid_thw[3 * i + 1]; grid[3 * j + 2] = grid_thw[3 * i + 2];
    }
    k = e;
  }
  if (epd_status stt = epd_encode(h, rows_scratch, cu.data(), (int32_t)miss.size(), grid.data(), (int32_t)miss.size(),
                                  out_scratch, stream)) return stt;
  size_t m0 = 0;
  for (size_t j = 0; j < miss.size(); ++j) {
    const int i = miss[j];
    const size_t bytes = (size_t)(mrg[i + 1] - mrg[i]) * row_bytes;
    const char* src = (const char*)out_scratch + m0 * row_bytes;
    EPD_HIP(h, hipMemcpyAsync((char*)out_visual_tokens + (size_t)mrg[i] * row_bytes, src, bytes, hipMemcpyDeviceToDevice, st));
    void* slot = nullptr;
    if (epd_store_insert(s, &keys[2 * i], bytes, &slot) == EPD_OK)
      EPD_HIP(h, hipMemcpyAsync(slot, src, bytes, hipMemcpyDeviceToDevice, st));
    m0 += (size_t)(mrg[i + 1] - mrg[i]);
  }
  return EPD_OK;
}

epd_status epd_encode_set_tuning(epd_handle h, int32_t gemm_tile, int32_t attn_groups) {
  if (!h) { g_create_error = "handle is NULL"; return EPD_ERR_INVALID_ARG; }
  if (gemm_tile != -1 && gemm_tile != 0 && gemm_tile != 2 && gemm_tile != 4 && gemm_tile != 5) {
    h->err = fmt("gemm_tile %d: -1 (automatic), 0, 2, 4 or 5", gemm_tile); return EPD_ERR_INVALID_ARG;
  }
  if (attn_groups < 0 || attn_groups > 2) { h->err = fmt("attn_groups %d: 0 (automatic), 1 or 2", attn_groups); return EPD_ERR_INVALID_ARG; }
  if (attn_groups && attn_q_tile(h->cfg.dtype == EPD_BF16, h->cfg.head_dim, 1, attn_groups) <= 0) {
    h->err = fmt("attn_groups %d has no kernel for head_dim %d", attn_groups, h->cfg.head_dim); return EPD_ERR_UNSUPPORTED;
  }
  h->tile_cfg = gemm_tile + 1;
  h->attn_groups = h->cfg.dtype == EPD_BF16 ? attn_groups : 0;
  return EPD_OK;
}

epd_status epd_encode_set_compute_units(epd_handle h, int32_t compute_units) {
  if (!h) { g_create_error = "handle is NULL"; return EPD_ERR_INVALID_ARG; }
  if (compute_units < 0 || compute_units > 4096) { h->err = fmt("compute_units %d: 0 (the whole device) or 1 .. 4096", compute_units); return EPD_ERR_INVALID_ARG; }
  h->compute_units = compute_units;
  return EPD_OK;
}

epd_status epd_encode_set_timing(epd_handle h, int32_t step) {
  if (!h) return EPD_ERR_INVALID_ARG;
  if (step < -1 || step >= EPD_STEP_COUNT) { h->err = "step out of range"; return EPD_ERR_INVALID_ARG; }
  h->timed_step = step;
  h->ev_used = 0;
  h->timed_work = 0.0;
  return EPD_OK;
}

epd_status epd_encode_get_timing(epd_handle h, double* total_ms, int64_t* launches, double* work) {
  if (!h || !total_ms || !launches) return EPD_ERR_INVALID_ARG;
  double ms = 0.0;
  for (int i = 0; i + 1 < h->ev_used; i += 2) {
    EPD_HIP(h, hipEventSynchronize(h->ev[i + 1]));
    float t = 0.f;
    EPD_HIP(h, hipEventElapsedTime(&t, h->ev[i], h->ev[i + 1]));
    ms += t;
  }
  *total_ms = ms;
  *launches = h->ev_used / 2;
  if (work) *work = h->timed_work;
  h->ev_used = 0;
  h->timed_work = 0.0;
  return EPD_OK;
}

}  // extern "C"
