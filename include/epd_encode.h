/* epd_encode.h -- C ABI of the MI355X (gfx950) Encode-stage library.
 *
 * The Encode stage of an Encode / Prefill / Decode disaggregated multimodal server maps a
 * multimodal input I_m to an embedding sequence V_m = E(I_m), V_m in R^{n x d}: n visual
 * tokens, one d-dimensional row each (paper section 3.1 "Encode Stage", Eq. 1).  For images
 * and video E is a Vision Transformer whose attention cost grows quadratically with the
 * visual sequence length (paper section 1).  This library is that forward pass:
 *
 *   packed patch rows -> patch embedding -> L x [norm, QKV + rotary, block-diagonal
 *   non-causal attention, output projection + residual, norm, GELU MLP + residual]
 *   -> final norm -> merge x merge spatial gather -> projection -> V_m.
 *
 * Every step runs in hand-written HIP kernels on the caller's stream.  The library never
 * allocates device memory: the caller provides one workspace (see
 * epd_encode_workspace_bytes) that also receives a repacked copy of the weights.
 *
 * Conventions
 *   - "device" pointers are HIP device memory on the current device, "host" pointers are
 *     ordinary process memory.  All matrices are dense row-major.
 *   - Linear weights are W[out, in] with bias b[out]; y = x W^T + b.
 *   - Status codes are returned, nothing aborts or throws across the ABI; a message for the
 *     last failure is available from epd_encode_last_error.  After any error the handle
 *     remains usable.
 *   - Execution is asynchronous on `stream`; kernel faults surface at the caller's next
 *     synchronisation.  One call at a time per handle (the workspace is shared).
 *   - Results are deterministic: identical inputs give bit-identical outputs (no atomics,
 *     no data-dependent reduction order), so a consumer that lost a feature can recompute
 *     it (paper section 3.2, fault-tolerant recomputation) and obtain the same tensor.
 */
#ifndef EPD_ENCODE_H
#define EPD_ENCODE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct epd_encoder* epd_handle;

typedef enum {
  EPD_MISS = 1,             /* epd_store_lookup only: key not present (not a failure)          */
  EPD_OK = 0,
  EPD_ERR_INVALID_ARG = -1, /* NULL pointer, bad enum value, bad struct_size            */
  EPD_ERR_UNSUPPORTED = -2, /* a shape the kernels do not cover (see epd_encode_create)  */
  EPD_ERR_SHAPE = -3,       /* per-call metadata inconsistent or over the configured max  */
  EPD_ERR_WORKSPACE = -4,   /* workspace missing, misaligned or too small                 */
  EPD_ERR_HIP = -5          /* a HIP runtime call failed (message has the HIP error)      */
} epd_status;

typedef enum { EPD_F32 = 0, EPD_BF16 = 1 } epd_dtype;
typedef enum { EPD_LAYERNORM = 0, EPD_RMSNORM = 1 } epd_norm;
typedef enum { EPD_GELU_ERF = 0, EPD_GELU_TANH = 1 } epd_act;
typedef enum { EPD_ROPE_NONE = 0, EPD_ROPE_2D = 2, EPD_ROPE_3D = 3 } epd_rope;

/* Per-layer tensors: DEVICE pointers, element type = cfg.dtype. */
typedef struct {
  const void* norm1_g; /* [D]                                                      */
  const void* norm1_b; /* [D], NULL for RMSNorm                                    */
  const void* qkv_w;   /* [3D, D]; rows: Q heads, then K heads, then V heads       */
  const void* qkv_b;   /* [3D] or NULL when use_bias == 0                          */
  const void* proj_w;  /* [D, D]                                                   */
  const void* proj_b;  /* [D] or NULL                                              */
  const void* norm2_g; /* [D]                                                      */
  const void* norm2_b; /* [D], NULL for RMSNorm                                    */
  const void* fc1_w;   /* [F, D]                                                   */
  const void* fc1_b;   /* [F] or NULL                                              */
  const void* fc2_w;   /* [D, F]                                                   */
  const void* fc2_b;   /* [D] or NULL                                              */
} epd_layer_weights;

typedef struct {
  const void* patch_w;             /* device [D, Pdim], Pdim = in_channels*temporal_patch*patch^2 */
  const void* patch_b;             /* device [D] or NULL                                           */
  const epd_layer_weights* layers; /* HOST array [num_layers] of device pointers                   */
  const void* final_norm_g;        /* device [D] (ignored when final_norm == 0)                    */
  const void* final_norm_b;        /* device [D], NULL for RMSNorm                                 */
  const void* merge_w;             /* device [out_dim, merge*merge*D]                              */
  const void* merge_b;             /* device [out_dim] or NULL                                     */
} epd_weights;

typedef struct {
  uint32_t struct_size; /* sizeof(epd_encode_cfg) of the caller's header (ABI check)            */
  int32_t dtype;        /* epd_dtype: storage type of weights, input patches and output.
                           EPD_F32 computes in true fp32; EPD_BF16 multiplies in bf16 on the
                           matrix cores with fp32 accumulation and an fp32 residual stream.    */
  int32_t num_layers;   /* L >= 0                                                              */
  int32_t hidden;       /* D = num_heads * head_dim                                            */
  int32_t num_heads;    /* H                                                                   */
  int32_t head_dim;     /* d, even; bf16: multiple of 8 and <= 128; fp32: <= 128               */
  int32_t mlp_dim;      /* F                                                                   */
  int32_t in_channels, patch, temporal_patch;
  int32_t norm;         /* epd_norm                                                            */
  float norm_eps;
  int32_t act;          /* epd_act                                                             */
  int32_t use_bias;     /* 1: every linear has a bias vector                                   */
  int32_t rope;         /* epd_rope                                                            */
  float rope_base;
  int32_t rope_pairs[3]; /* rotary pairs of the (t, h, w) axes; sum = head_dim/2 unless
                            rope == EPD_ROPE_NONE.  Pair p of a head is its elements
                            (p, p + d/2); pairs go to the axes in the order t, h, w; the
                            j-th pair of an axis with n pairs turns by coord * base^(-j/n). */
  int32_t final_norm;   /* 1: norm before the merger                                           */
  int32_t merge;        /* spatial merge size m (2; 1 = no gather)                             */
  int32_t out_dim;      /* width of V_m                                                        */
  int32_t max_tokens;   /* largest T (packed patch rows) of any call; bf16: max_tokens *
                           hidden < 2^30 (EPD_ERR_UNSUPPORTED beyond)                          */
  int32_t max_segments; /* largest number of attention segments of any call                    */
  int32_t max_items;    /* largest number of images / clips of any call                        */
  const epd_weights* weights; /* HOST struct of device pointers; read (copied into the
                                 workspace in kernel-friendly order) during create, free to
                                 release afterwards                                            */
  void* workspace;      /* device, 256-byte aligned, >= epd_encode_workspace_bytes(cfg);
                           owned by the caller, must outlive the handle                        */
  uint64_t workspace_bytes;
} epd_encode_cfg;

/* Bytes of device workspace a handle for `cfg` needs (weights copy + activations + plan
 * arrays).  Pure host arithmetic; only the shape fields of cfg are read.  Returns 0 when
 * cfg is NULL or invalid. */
uint64_t epd_encode_workspace_bytes(const epd_encode_cfg* cfg);

/* Build an encoder E (Eq. 1).  Validates cfg (EPD_ERR_INVALID_ARG / EPD_ERR_UNSUPPORTED /
 * EPD_ERR_WORKSPACE are decided on the host before any HIP call), copies and reorders the
 * weights into the workspace on the null stream and waits for that copy.  *out is written
 * only on success. */
epd_status epd_encode_create(const epd_encode_cfg* cfg, epd_handle* out);

/* V_m = E(I_m).
 *   packed_patches    device [T, Pdim], cfg.dtype.  Items (images / clips) are packed in
 *                     order; item (t, h, w) contributes t*h*w rows in raster order
 *                     (ti*h + r)*w + c; a row holds (channel, temporal offset, row in
 *                     patch, column in patch).
 *   cu_seqlens        HOST int32 [num_segments + 1]: attention segment s is the token range
 *                     [cu[s], cu[s+1]); cu[0] = 0, strictly increasing, cu[last] = T.
 *                     A token attends to the tokens of its own segment only (non-causal).
 *   grid_thw          HOST int32 [num_items, 3]: (t, h, w) in patch units; sum t*h*w = T;
 *                     h and w divisible by cfg.merge.  Rotary coordinates are (ti, r, c)
 *                     within the item.  Segments need not coincide with items.
 *   out_visual_tokens device [sum t*(h/m)*(w/m), out_dim], cfg.dtype: merged token
 *                     (ti, i, j) concatenates window rows then columns
 *                     ((mi, mj), (mi, mj+1), ..., (mi+1, mj), ...) and is projected.
 *   stream            hipStream_t (NULL = the null stream).
 * Both host arrays are consumed before the call returns.  Inconsistent metadata returns
 * EPD_ERR_SHAPE with nothing launched. */
epd_status epd_encode(epd_handle h, const void* packed_patches, const int32_t* cu_seqlens,
                      int32_t num_segments, const int32_t* grid_thw, int32_t num_items,
                      void* out_visual_tokens, void* stream);

/* I_m -> packed patch rows: the step in front of epd_encode (section 3.1: the Encode stage
 * receives the raw multimodal input I_m, images and video; Eq. 1).  The paper does not say how
 * I_m becomes encoder input; this library fixes: every frame is resized to the item's grid,
 * (h * patch) x (w * patch) pixels, by bilinear interpolation with half-pixel centres and the
 * source coordinate clamped to the image (no antialiasing filter, frames are not resampled in
 * time, equal sizes copy pixels unchanged); values become (v / 255 - mean[c]) / std[c]; rows
 * are laid out as epd_encode expects them.
 *   pixels          device uint8: items packed in order, item i planar
 *                   [in_channels, t_i * temporal_patch, Hs_i, Ws_i]
 *   src_hw          HOST int32 [num_items, 2]: (Hs_i, Ws_i), 1 .. 16384 each
 *   grid_thw        HOST int32 [num_items, 3]: (t, h, w) in patch units; sum t*h*w <= max_tokens
 *   mean, std       HOST float [in_channels] on the 0..1 pixel scale; std > 0
 *   packed_patches  device [sum t*h*w, Pdim], cfg.dtype (output; at least 8-byte aligned)
 *   stream          hipStream_t (NULL = the null stream)
 * Uses cfg's in_channels (<= 8), patch (even, <= 32), temporal_patch and dtype; allocates nothing and
 * touches neither the workspace nor a running epd_encode.  The host arrays are consumed before
 * the call returns.  Bad metadata returns EPD_ERR_SHAPE / EPD_ERR_INVALID_ARG /
 * EPD_ERR_UNSUPPORTED with nothing launched. */
epd_status epd_preprocess(epd_handle h, const uint8_t* pixels, const int32_t* src_hw,
                          const int32_t* grid_thw, int32_t num_items, const float* mean,
                          const float* std, void* packed_patches, void* stream);

/* ---- single-node stand-in for the MM Store (section 3.2) -------------------------------
 * "Multimodal Cache Pooling": encoded features are stored under the hash of the multimodal
 * input, so that a repeated input is not encoded again; "Fault-Tolerant and Recomputation": a
 * feature that cannot be fetched is recomputed.  The paper names neither the hash nor the
 * pool's replacement rule; this library fixes:
 *   key    two polynomial hashes modulo P = 2^61 - 1 with bases R_0 = 0x1D4E2C1B3A596877 mod P,
 *          R_1 = 0x0F1E2D3C4B5A6978 mod P over the words s_0 .. s_{L-1} = byte length (low,
 *          high 32 bits), salt (low, high), then the input as 32-bit little-endian words (last
 *          one zero-padded):  H_k = sum_j (s_j + 1) * R_k^(L - j) mod P.
 *   pool   caller-owned device memory; the first 1 MiB is scratch for the hash, the rest an
 *          arena of contiguous, 256-byte aligned entries; an insert drops least-recently-used
 *          entries until a free range (first fit, lowest address) holds the new entry; a
 *          lookup that hits makes its entry the most recent.
 * One call per store at a time.  Bookkeeping (create / lookup / insert / stats / destroy) is
 * host code and never touches device memory. */
typedef struct epd_store* epd_store_handle;

/* device_pool: device, 256-byte aligned, pool_bytes > 1 MiB; owned by the caller, must outlive
 * the store.  *out is written only on success. */
epd_status epd_store_create(void* device_pool, uint64_t pool_bytes, epd_store_handle* out);
epd_status epd_store_destroy(epd_store_handle s);
/* Message of the last failure on this store (of the last failed create when s == NULL). */
const char* epd_store_last_error(epd_store_handle s);

/* Keys of n byte ranges of one device buffer: range i = [offsets[i], offsets[i+1]) (HOST
 * uint64 [n + 1], non-decreasing, each range < 8 GiB), salts HOST uint64 [n], keys_out HOST
 * uint64 [n, 2].  Launches on `stream` and waits for the keys. */
epd_status epd_store_hash(epd_store_handle s, const void* device_data, const uint64_t* offsets,
                          const uint64_t* salts, int32_t n, uint64_t* keys_out, void* stream);

/* For callers that cannot allocate device memory or wait for the GPU -- code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc: the keys of epd_store_hash (bit
 * for bit), with no store, no pool and no host synchronisation.
 *   device_data      device: the buffer the ranges lie in
 *   offsets, salts   HOST uint64 [n + 1] / [n], as for epd_store_hash; consumed before the call returns
 *   n                1 .. 32 ranges per call; more returns EPD_ERR_SHAPE with nothing launched
 *   keys_device_out  DEVICE uint64 [n, 2]: written by the second of the two kernels this call
 *                    enqueues on `stream`; valid once the stream has passed that kernel
 * The partial hashes live in a 512 KiB array the library holds statically on every GPU it is
 * loaded on (one copy per GPU, for the life of the process): the call allocates and frees nothing,
 * copies nothing and waits for nothing.  All calls on one GPU share that array, so two calls whose
 * kernels may overlap on the same GPU (different streams) race: order them.  Calls on different
 * GPUs are independent.  Errors: EPD_ERR_INVALID_ARG (NULL pointer, n <= 0), EPD_ERR_SHAPE (n > 32,
 * decreasing offsets, a range of 8 GiB or more), EPD_ERR_HIP; message from
 * epd_store_last_error(NULL). */
epd_status epd_store_hash_noalloc(const void* device_data, const uint64_t* offsets,
                                  const uint64_t* salts, int32_t n, uint64_t* keys_device_out,
                                  void* stream);

/* EPD_OK: *device_ptr / *bytes describe the stored value (valid until a later insert drops
 * it); EPD_MISS: not stored.  `bytes` may be NULL. */
epd_status epd_store_lookup(epd_store_handle s, const uint64_t key[2], void** device_ptr,
                            uint64_t* bytes);
/* Reserve `bytes` for `key` (replacing an entry of the same key) and return where the caller
 * must write the value, in stream order before any reader.  EPD_ERR_WORKSPACE (nothing
 * dropped) when the entry can never fit. */
epd_status epd_store_insert(epd_store_handle s, const uint64_t key[2], uint64_t bytes,
                            void** device_ptr);
/* Counters since create; any pointer may be NULL. */
epd_status epd_store_stats(epd_store_handle s, uint64_t* hits, uint64_t* misses,
                           uint64_t* evictions, uint64_t* entries);

/* V_m = E(I_m) through the store: every item (image / clip) is keyed by the hash of its pixels,
 * salted with its source size, grid, the patch geometry, dtype and `model_salt` (which must
 * identify the weights):  x = model_salt; for f in (Hs, Ws, t, h, w, patch, temporal_patch,
 * in_channels, dtype): x = (x ^ (uint64)f) * 0x9E3779B97F4A7C15 mod 2^64.  Items found in the
 * store are copied from it; the others are preprocessed (epd_preprocess), encoded together in
 * one epd_encode call with one attention segment per item, filed in the store and copied to
 * their rows of out_visual_tokens.  Arguments as in epd_preprocess / epd_encode, plus
 *   rows_scratch   device [sum t*h*w, Pdim], cfg.dtype: patch rows of the items that miss
 *   out_scratch    device [sum merged tokens, out_dim], cfg.dtype: their rows before filing
 *   hit_out        HOST int32 [num_items] or NULL: 1 = served from the store
 *   keys_out       HOST uint64 [num_items, 2] or NULL
 * Waits on `stream` once (for the keys); everything else is asynchronous on it.  An item too
 * large for the pool is encoded and returned but not stored. */
epd_status epd_encode_cached(epd_handle h, epd_store_handle s, uint64_t model_salt,
                             const uint8_t* pixels, const int32_t* src_hw,
                             const int32_t* grid_thw, int32_t num_items, const float* mean,
                             const float* std, void* rows_scratch, void* out_scratch,
                             void* out_visual_tokens, int32_t* hit_out, uint64_t* keys_out,
                             void* stream);

/* Release host-side state (events, pinned staging).  The workspace stays the caller's. */
epd_status epd_encode_destroy(epd_handle h);

/* Message of the last failure on this handle (or of the last failed create on this thread
 * when h == NULL).  Never NULL; valid until the next call on the same handle / thread. */
const char* epd_encode_last_error(epd_handle h);

/* ---- measurement and test hooks (not needed to serve) --------------------------------- */

/* Copy the fp32 residual stream [T, D] of the last epd_encode (the hidden state before the
 * final norm) to a device buffer, asynchronously on `stream`. */
epd_status epd_encode_debug_hidden(epd_handle h, void* out_T_by_D_f32, void* stream);

/* Tuning and test hook: force one variant of the bf16 kernels for all following epd_encode calls
 * of this handle (ignored by the fp32 path).
 *   gemm_tile    -1 = the library's choice per GEMM; 0 (256x256), 2 (256x128), 4 (128x128) or
 *                5 (320x256) = that output tile for every GEMM that can take it
 *   attn_groups  0 = the library's choice; 1 = 128, 2 = 256 query rows per block of the attention
 *                kernel (256: two 32-row groups per wave for head_dim <= 64, eight waves of one
 *                group for larger head dims); EPD_ERR_UNSUPPORTED where a setting has no kernel
 * Any other value returns EPD_ERR_INVALID_ARG and changes nothing.  Results stay within the
 * stated tolerances under every setting; they are bit-identical only under the same setting. */
epd_status epd_encode_set_tuning(epd_handle h, int32_t gemm_tile, int32_t attn_groups);

/* Co-location (section 3.5, "Physical Co-Location and Spatial Multiplexing": stages share one
 * device): tell the handle that its following epd_encode calls run on a stream that is masked to
 * `compute_units` compute units (hipExtStreamCreateWithCUMask), so that the GEMM launcher counts
 * its rounds of tiles for that many units instead of the whole device -- a stream's mask is not
 * visible to the library.  0 = the whole device (the default).  Changes the launch plans only,
 * never a result beyond rounding.  EPD_ERR_INVALID_ARG outside 0 .. 4096 or on a NULL handle. */
epd_status epd_encode_set_compute_units(epd_handle h, int32_t compute_units);

/* Steps of the path, for per-kernel timing. */
typedef enum {
  EPD_STEP_PLAN = 0, EPD_STEP_PATCH_EMBED = 1, EPD_STEP_NORM = 2, EPD_STEP_QKV = 3,
  EPD_STEP_ATTN = 4, EPD_STEP_PROJ = 5, EPD_STEP_FC1 = 6, EPD_STEP_FC2 = 7,
  EPD_STEP_MERGE = 8, EPD_STEP_COUNT = 9
} epd_step;

/* Bracket every launch of `step` (an epd_step, or -1 to switch timing off) with HIP events
 * on the stream it is launched on, in all following epd_encode calls. */
epd_status epd_encode_set_timing(epd_handle h, int32_t step);

/* Wait for the recorded events, return the summed kernel time and launch count since the
 * last call of this function, and clear them.  Also returns the algorithmic work of those
 * launches (flops for matrix steps, bytes moved for the norm step). */
epd_status epd_encode_get_timing(epd_handle h, double* total_ms, int64_t* launches,
                                 double* work);

/* Synthetic memory-bound neighbour for the co-location experiment (section 3.5: stages with
 * dissimilar resource demands share one device): one launch streams device_buf[0, bytes) once
 * (16-byte loads, bytes rounded down to a multiple of 16, buffer 16-byte aligned) with `blocks`
 * blocks of 256 threads (1 .. 65536) and writes one value per block to device_out[blocks].
 * Asynchronous on `stream`; allocates nothing.  EPD_ERR_INVALID_ARG on a NULL or misaligned
 * pointer, bytes < 16 or a block count out of range. */
epd_status epd_probe_stream_read(const void* device_buf, uint64_t bytes, float* device_out,
                                 int32_t blocks, void* stream);

/* Matrix-core rate on register-resident operands (no memory traffic): the practical ceiling of
 * the bf16 matrix pipes under the chip's power limit, which depends on the operand values.
 *   shape          0 = v_mfma_f32_32x32x16_bf16 (the attention kernel's instruction),
 *                  1 = v_mfma_f32_16x16x32_bf16 (the GEMMs')
 *   zero_operands  0 = random operands of magnitude [0.5, 1), 1 = all-zero operands
 *   iters          loop trips per wave (> 0)
 *   device_out     device float [256 * 512]: one value per thread (keeps the work observable)
 *   flops_per_launch  HOST out (may be NULL): flops one launch executes
 * Launches 256 blocks of 512 threads on `stream`; allocates nothing.  EPD_ERR_INVALID_ARG on a bad
 * shape, iters <= 0 or a NULL output. */
epd_status epd_probe_mfma_rate(int32_t shape, int32_t zero_operands, int32_t iters,
                               float* device_out, double* flops_per_launch, void* stream);

/* Host only, launches nothing: how the bf16 GEMM of the encoder layers would tile an M x N
 * output (tokens x output columns) with inner dimension K on a chip of `compute_units` units
 * (<= 0: the current device's, 256 where there is none).  The layer GEMMs of V_m = E(I_m)
 * (section 3.1, Eq. 1) run as one launch of tile_rows x tile_cols tiles, or -- body_rows > 0 --
 * as that launch over the first body_rows tokens plus a second launch of 128 x 128 tiles over the
 * rest, which turns a partial last round of large tiles into a round of small ones.
 *   epilogue  0 = store, 1 = GELU (first MLP GEMM), 2 = residual add (attention output projection,
 *             second MLP GEMM), 3 = the QKV projection (Q | K columns [0, qk_cols), then V)
 * All three outputs are HOST pointers.  EPD_ERR_INVALID_ARG on M, N, K <= 0, an epilogue outside
 * 0 .. 3, a NULL output, or qk_cols outside (0, N] with epilogue 3. */
epd_status epd_probe_gemm_plan(int32_t M, int32_t N, int32_t K, int32_t epilogue, int32_t qk_cols,
                               int32_t compute_units, int32_t* tile_rows, int32_t* tile_cols,
                               int32_t* body_rows);

#ifdef __cplusplus
}
#endif
#endif /* EPD_ENCODE_H */
