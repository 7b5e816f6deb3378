/*
 * nova.h -- C ABI of the MI355X (gfx950) hot path of NOVA's entropy-guided token
 * reduction for visual autoregressive (next-scale prediction) transformers.
 *
 * One transformer block at one next-scale step is four calls:
 *   nova_entropy      token predictive entropy of the codebook logits
 *   nova_select       keep the k highest-entropy tokens of every batch row
 *   nova_pruned_block attention + FFN on the kept tokens only
 *   nova_merge_cache  scatter back; pruned tokens reuse the upsampled residual cache
 *
 * Conventions (all entry points):
 *   - Every data pointer is a DEVICE pointer unless its comment says "host".
 *     The caller owns every buffer; the library allocates nothing, frees
 *     nothing and never synchronises.  All work is enqueued on `stream`
 *     (a hipStream_t passed as void*; NULL = the default stream).
 *   - Inputs are read-only; outputs must not alias inputs.
 *   - Arrays are dense row-major unless a stride argument says otherwise.
 *   - Return value: NOVA_OK (0) or a negative NOVA_ERR_* code.  Argument
 *     errors are detected on the host before anything is launched and leave
 *     the outputs untouched.  Nothing is printed, nothing aborts.
 *   - A context is bound to one device; use one context per host thread.
 */
#ifndef NOVA_H
#define NOVA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  NOVA_OK = 0,
  NOVA_ERR_INVALID_ARG = -1, /* null pointer, negative size, k > N, misaligned pointer ...      */
  NOVA_ERR_UNSUPPORTED = -2, /* valid request the kernels do not cover (dtype, head size ...)  */
  NOVA_ERR_WORKSPACE = -3,   /* workspace smaller than nova_workspace_bytes()                   */
  NOVA_ERR_HIP = -4,         /* a HIP runtime call failed (launch error, wrong device ...)      */
  NOVA_ERR_STATIC_SCRATCH = -5 /* the request needs more than the static scratch of the allocation-free entry point */
};

enum { NOVA_F32 = 0, NOVA_BF16 = 1 }; /* storage type of activations / weights / logits */

typedef struct nova_ctx nova_ctx;

/* Shape of one pruned block call.  F = ffn_mult * C is the FFN hidden width. */
typedef struct nova_block_shape {
  int32_t dtype;       /* NOVA_F32 or NOVA_BF16: x, weights, caches, outputs           */
  int32_t B;           /* batch rows (images)                                            */
  int32_t N;           /* tokens of the current scale per batch row (h*w)                */
  int32_t C;           /* model width                                                    */
  int32_t heads;       /* attention heads; dh = C / heads                                */
  int32_t ffn_mult;    /* FFN expansion (4 in every workload here)                       */
  int32_t kv_len;      /* P: rows already in the KV cache (all prior scales)             */
  int32_t kv_capacity; /* rows allocated per (batch row, head) in the caches, >= P + k   */
  int32_t k;           /* kept tokens per batch row, 0 <= k <= N                         */
} nova_block_shape;

/* Block weights, device pointers, same dtype as the activations.  Matrices are
 * stored out-feature major: W[out][in], so a projection is y = u * W^T + b.
 * Biases may be NULL (treated as zero).  Every non-NULL pointer must be 16-byte aligned. */
typedef struct nova_block_weights {
  const void* w_qkv; /* [3C, C]  rows 0..C-1 query, C..2C-1 key, 2C..3C-1 value */
  const void* b_qkv; /* [3C]                                                     */
  const void* w_o;   /* [C, C]                                                   */
  const void* b_o;   /* [C]                                                      */
  const void* w_fc1; /* [F, C]                                                   */
  const void* b_fc1; /* [F]                                                      */
  const void* w_fc2; /* [C, F]                                                   */
  const void* b_fc2; /* [C]                                                      */
} nova_block_weights;

/* Variations of the block that the backbones of Sec. 4 differ in (all off = the block documented at
 * nova_pruned_block).  The paper names the backbones, not these details; the formulas are this library's.
 *   gelu_tanh  0: erf GELU; 1: 0.5 v (1 + tanh(sqrt(2/pi) (v + 0.044715 v^3)))
 *   qk_norm    0 | 1.  1: per head, q <- q / max(|q|, 1e-12), kk <- kk / max(|kk|, 1e-12) (Euclidean
 *              length over dh), scores = qk_scale[head] * <q, k> instead of <q, k> / sqrt(dh); the rows
 *              appended to k_cache are the unit-length keys and rows [0, P) are taken to be such rows
 *   qk_scale   DEVICE fp32 [heads]; required when qk_norm, ignored otherwise
 *   ada        NULL, or DEVICE [B, 6, C] in the activations' dtype, 16-byte aligned: per image
 *              (shift1, scale1, gate1, shift2, scale2, gate2), used as
 *                u  = LN(xs) (1 + scale1) + shift1        x1     = xs + gate1 * (a W_o^T + b_o)
 *                u2 = LN(x1) (1 + scale2) + shift2        y_kept = x1 + gate2 * (GELU(u2 W_fc1^T + b_fc1) W_fc2^T + b_fc2)
 *   w_cq ...   a cross-attention sub-layer over `text_len` condition tokens, between the self-attention
 *              branch and the FFN branch (w_cq == NULL: none):
 *                x1 <- x1 + softmax((LN(x1) w_cq^T + b_cq) Kt^T / sqrt(dh)) Vt w_co^T + b_co   per head
 *              w_cq, w_co  DEVICE [C, C] out-feature major;  b_cq, b_co  DEVICE [C] or NULL
 *              k_text      DEVICE [B, heads, text_capacity, dh]  projected keys of the condition tokens,
 *              v_text      DEVICE [B, heads, dh, text_capacity]  projected values, token index minor
 *                          (the layouts of k_cache / v_cache); rows / columns [0, text_len) are read
 *              1 <= text_len <= text_capacity; NOVA_BF16: text_capacity % 64 == 0; NOVA_F32: text_len + dh <= 16384.
 *              All in the activations' dtype, 16-byte aligned.  Neither qk_norm nor the gates apply to it.
 */
typedef struct nova_block_variant {
  int32_t gelu_tanh;
  int32_t qk_norm;
  const float* qk_scale;
  const void* ada;
  const void* w_cq;
  const void* b_cq;
  const void* w_co;
  const void* b_co;
  const void* k_text;
  const void* v_text;
  int32_t text_len;
  int32_t text_capacity;
} nova_block_variant;

/* Creates a context for HIP device `device_id` (queries its properties).
 * *out is a host object owned by the caller; release with nova_destroy. */
int nova_create(nova_ctx** out, int device_id);
int nova_destroy(nova_ctx* ctx);

/* Static description of an error code (host string, never NULL). */
const char* nova_strerror(int code);

/* Bytes of device workspace nova_pruned_block needs for `shape` (0 if k == 0 or the
 * shape is invalid).  The workspace holds intermediates only; contents are undefined
 * between calls. */
size_t nova_workspace_bytes(const nova_block_shape* shape);

/*
 * Token predictive entropy (Sec. 3.3, "Adaptive Acceleration Activation", the
 * entropy equation): for each of the batch*rows_per_batch tokens,
 *   H = -sum_v p(v) ln p(v),  p = softmax(logits[token, 0..V-1]),  natural log,
 * accumulated in fp32, written as fp32 (tiny negative rounding results are
 * clamped to +0).  A row containing NaN yields NaN.
 *   logits           [batch*rows_per_batch, V], row r starts at element
 *                    r*row_stride_elems (row_stride_elems >= V); dtype NOVA_F32|NOVA_BF16
 *   entropy          out [batch*rows_per_batch] fp32
 *   mean_entropy     out [batch] fp32 or NULL: the scale mean entropy of the same
 *                    section (mean over the rows_per_batch tokens of a batch row), summed in a
 *                    fixed order by a second small kernel: the same bits on every run.
 * batch == 0 or rows_per_batch == 0 is a no-op.  V >= 1.
 */
int nova_entropy(nova_ctx* ctx, void* stream, const void* logits, int logits_dtype,
                 int64_t rows_per_batch, int batch, int V, int64_t row_stride_elems,
                 float* entropy, float* mean_entropy);

/*
 * Token entropy of a bitwise token head (a token is d independent binary choices, as in the
 * Infinity backbones of Sec. 4; entropy equation of Sec. 3.3 on the product distribution):
 *   entropy[token] = sum_{i<d} h(softmax(bit_logits[token, i, 0], bit_logits[token, i, 1]))
 * with h the binary entropy in nats, evaluated in fp32.  NaN logits give NaN.
 *   bit_logits    [batch*rows_per_batch, d, 2] contiguous; dtype NOVA_F32 | NOVA_BF16
 *   entropy       out [batch*rows_per_batch] fp32;  mean_entropy out [batch] fp32 or NULL
 * d >= 1.  batch == 0 or rows_per_batch == 0 is a no-op.
 */
int nova_entropy_bits(nova_ctx* ctx, void* stream, const void* bit_logits, int logits_dtype,
                      int64_t rows_per_batch, int batch, int d, float* entropy, float* mean_entropy);

/*
 * Token entropy straight from a linear prediction head (Sec. 4, "Entropy Computation
 * Overhead": the distributions are the ones decoding produces; entropy equation of Sec. 3.3):
 *   logits = hidden W_head^T + b_head   (fp32 accumulation on the matrix cores, never stored)
 *   entropy[token] = -sum_v p(v) ln p(v),  p = softmax(logits[token, :])
 * i.e. nova_entropy of the head's output without the [tokens, V] logits round trip through HBM.
 *   hidden        [batch*rows_per_batch, C]  NOVA_BF16 (the only dtype supported), C % 64 == 0
 *   w_head        [V, C] out-feature major;  b_head [V] or NULL
 *   entropy       out [batch*rows_per_batch] fp32;  mean_entropy out [batch] fp32 or NULL
 *   workspace     device scratch of at least nova_head_entropy_workspace_bytes(...), 16-byte aligned
 * Inputs must be finite.  The logits differ from bf16-stored ones by that rounding, so the result
 * agrees with nova_entropy on stored logits only to the storage precision; against exact
 * arithmetic on the same inputs |dH| <= 1e-4 |H| + 1e-5.
 */
size_t nova_head_entropy_workspace_bytes(int64_t rows_per_batch, int batch, int V);
int nova_head_entropy(nova_ctx* ctx, void* stream, const void* hidden, const void* w_head,
                      const void* b_head, int dtype, int64_t rows_per_batch, int batch, int C, int V,
                      float* entropy, float* mean_entropy, void* workspace, size_t workspace_bytes);

/*
 * nova_head_entropy for callers that cannot allocate device memory or pass a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same kernels, with the per-tile entropy
 * partials in a static device array of NOVA_HEAD_ENTROPY_STATIC_BYTES (4 MiB) that each GPU the library runs
 * on holds until the process ends (its address on the context's device is resolved by nova_create).  The call
 * allocates nothing.  It needs 16 bytes per row and per column tile of the GEMM configuration picked for the
 * shape (256 columns at the large workloads: 2 MiB for 8192 rows and V = 4096); a request that needs more than
 * the array returns NOVA_ERR_STATIC_SCRATCH and launches nothing.  Results are those of nova_head_entropy, bit for
 * bit.  All calls on one GPU share the array: calls that overlap on one GPU (two streams, two threads, two contexts)
 * race; nothing in it has to be cleared between calls (every partial that is read is written first).
 */
#define NOVA_HEAD_ENTROPY_STATIC_BYTES ((size_t)4 << 20)
int nova_head_entropy_static(nova_ctx* ctx, void* stream, const void* hidden, const void* w_head,
                             const void* b_head, int dtype, int64_t rows_per_batch, int batch, int C, int V,
                             float* entropy, float* mean_entropy);

/*
 * Entropy-guided token selection (Sec. 3.3, "Dual-Linkage Acceleration", final
 * sentence: the lowest-entropy tokens are pruned at the reduction ratio; Sec. 3.2:
 * the highest-entropy tokens are maintained).  For each batch row the k tokens
 * first in the order (entropy descending, index ascending) are kept; the compare
 * is numeric on fp32 (-0 == +0) and NaN ranks below every number.
 *   entropy    [B, N] fp32
 *   k          kept tokens per row when k_per_row is NULL; 0 <= k <= N
 *   k_per_row  NULL, or DEVICE int32 [B]: per-row keep counts (clamped to [0, N] on
 *              the device); then `k` must be >= every count and is the row pitch of kept_idx
 *   kept_idx   out int32 [B, k]: kept token indices, ascending; entries past a row's
 *              count are set to -1
 *   keep_mask  out uint8 [B, N]: 1 = kept, 0 = pruned
 * N <= 65536.  B == 0 is a no-op.  The result is exact (integer compares on the
 * float bit patterns): identical to a stable sort.
 */
int nova_select(nova_ctx* ctx, void* stream, const float* entropy, int B, int N, int k,
                const int32_t* k_per_row, int32_t* kept_idx, uint8_t* keep_mask);

/*
 * One transformer block on the kept tokens only (Sec. 3.3, "Residual Cache Reuse",
 * first equation: R_out = Layer_j(R_in), evaluated for the kept rows; Sec. 3.2: pruning
 * reduces the attention cost).  With xs = x[b, kept_idx[b, s], :] for s = 0..k-1:
 *   u        = LN(xs)                       LayerNorm over C, no affine, eps 1e-6
 *   [q|kk|vv]= u W_qkv^T + b_qkv            kk, vv are appended to the caches at row P+s
 *   a        = per head softmax(q K^T / sqrt(dh)) V over the P+k cached rows (no mask)
 *   x1       = xs + a W_o^T + b_o
 *   y_kept   = x1 + GELU(LN(x1) W_fc1^T + b_fc1) W_fc2^T + b_fc2      (erf GELU)
 * The paper does not define Layer_j; this block structure is this library's.
 *   x        [B, N, C]
 *   kept_idx [B, k] int32, values in [0, N) (as written by nova_select)
 *   k_cache  [B, heads, kv_capacity, dh]   keys,   row-per-key; rows [0,P) are read,
 *                                          rows [P, P+k) are WRITTEN, others untouched
 *   v_cache  [B, heads, dh, kv_capacity]   values, key index minor (transposed so the
 *                                          P.V matrix-core operand is one 16-byte read);
 *                                          columns [0,P) read, [P,P+k) WRITTEN
 *   y_kept   out [B, k, C]
 *   workspace  device scratch of at least nova_workspace_bytes(shape), 256-byte aligned
 * NOVA_BF16 requires C % 64 == 0, dh in {64, 128}, kv_capacity % 64 == 0;
 * NOVA_F32 requires dh <= 256.  k == 0 is a no-op.
 */
int nova_pruned_block(nova_ctx* ctx, void* stream, const nova_block_shape* shape,
                      const nova_block_weights* weights, const void* x, const int32_t* kept_idx,
                      void* k_cache, void* v_cache, void* y_kept, void* workspace,
                      size_t workspace_bytes);

/* nova_pruned_block with the block variations of `variant` (NULL = none: identical to
 * nova_pruned_block).  Every other argument, requirement and error is as documented there;
 * a non-zero flag other than 1 or a missing qk_scale is NOVA_ERR_INVALID_ARG. */
int nova_pruned_block_variant(nova_ctx* ctx, void* stream, const nova_block_shape* shape,
                              const nova_block_weights* weights, const nova_block_variant* variant,
                              const void* x, const int32_t* kept_idx, void* k_cache, void* v_cache,
                              void* y_kept, void* workspace, size_t workspace_bytes);

/*
 * nova_pruned_block_variant with per-image keep counts on the device (Sec. 3.3, "Dual-Linkage Acceleration": the
 * scale- and layer-linkage ratios are per instance, so the images of a batch keep different numbers of tokens),
 * so that nova_layer_ratio -> nova_select -> this call -> nova_merge_cache_rows run without a host round trip.
 *   shape->k          row pitch: kept_idx is [B, k], y_kept [B, k, C], and no image keeps more (k = N is always safe).
 *                     Launch sizes and the workspace follow this k; output tiles and query blocks that hold no
 *                     live row leave at once, so the work done follows the counts.
 *   k_per_row         DEVICE int32 [B] or NULL (= k for every image): image b keeps the tokens kept_idx[b, 0 ..
 *                     k_per_row[b]) (clamped to [0, k]); the rest of its row is ignored (nova_select writes -1 there)
 *   shape->kv_len     upper bound of the images' prior-row counts; shape->kv_len + shape->k <= kv_capacity
 *   kv_len_per_row    DEVICE int32 [B] or NULL (= kv_len for every image): rows already in image b's K/V cache
 *                     (clamped to [0, kv_len]).  Image b attends to those rows plus its own kept rows, which are
 *                     appended right behind them.
 *   kv_len_next       DEVICE int32 [B] or NULL: receives kv_len_per_row[b] + k_per_row[b], the image's cache length
 *                     after this block; may be the kv_len_per_row array itself (it is written after every read)
 *   y_kept            rows [b, s] with s >= k_per_row[b] are undefined (some are never written)
 * Every image's result is that of a single-image call with its own counts.  Everything else (variant may be NULL)
 * as nova_pruned_block_variant.  The three count arrays must be 4-byte aligned.
 */
int nova_pruned_block_rows(nova_ctx* ctx, void* stream, const nova_block_shape* shape,
                           const nova_block_weights* weights, const nova_block_variant* variant,
                           const int32_t* k_per_row, const int32_t* kv_len_per_row, int32_t* kv_len_next,
                           const void* x, const int32_t* kept_idx, void* k_cache, void* v_cache, void* y_kept,
                           void* workspace, size_t workspace_bytes);

/*
 * Residual cache reuse (Sec. 3.3, "Residual Cache Reuse", second and third equations):
 *   cache_up   = bilinear upsample of cache_prev from the (hp, wp) grid to (h, w),
 *                half-pixel centres, evaluated in fp32
 *   out[b,i]   = y_kept[b,s]              if i == kept_idx[b,s]   (copied bit for bit)
 *              = x[b,i] + cache_up[b,i]   otherwise               (one rounding)
 *   cache_new[b,i] = out[b,i] - x[b,i]    (for pruned rows this is cache_up itself)
 *   x          [B, h*w, C]      block input
 *   y_kept     [B, k, C]        nova_pruned_block output (unused if k == 0)
 *   kept_idx   [B, k] int32 ascending, keep_mask [B, h*w] uint8 (from nova_select)
 *   cache_prev [B, hp*wp, C]    residual cache of the prior scale; may be NULL iff k == h*w
 *   out        [B, h*w, C]      must not alias x
 *   cache_new  [B, h*w, C] or NULL
 * dtype NOVA_F32 | NOVA_BF16 applies to x, y_kept, cache_prev, out, cache_new.
 */
int nova_merge_cache(nova_ctx* ctx, void* stream, int dtype, int B, int C, int h, int w, int hp,
                     int wp, int k, const void* x, const void* y_kept, const int32_t* kept_idx,
                     const uint8_t* keep_mask, const void* cache_prev, void* out, void* cache_new);

/*
 * nova_merge_cache with another interpolation kernel for cache_up (the paper says only that the cache
 * is interpolated to the next scale's grid; bilinear is this library's default reading):
 *   NOVA_INTERP_BILINEAR  as nova_merge_cache
 *   NOVA_INTERP_NEAREST   the source cell containing the output cell's centre:
 *                         index min(floor((i + 1/2) n_in / n_out), n_in - 1) per axis, exact
 *   NOVA_INTERP_BICUBIC   separable cubic convolution with kernel parameter a = -3/4, half-pixel
 *                         centres, taps floor(src) - 1 .. floor(src) + 2 clamped to the grid, fp32
 * Any other value of `interp` is NOVA_ERR_INVALID_ARG.  Everything else as nova_merge_cache.
 */
enum { NOVA_INTERP_BILINEAR = 0, NOVA_INTERP_NEAREST = 1, NOVA_INTERP_BICUBIC = 2 };
int nova_merge_cache_interp(nova_ctx* ctx, void* stream, int dtype, int interp, int B, int C, int h, int w,
                            int hp, int wp, int k, const void* x, const void* y_kept, const int32_t* kept_idx,
                            const uint8_t* keep_mask, const void* cache_prev, void* out, void* cache_new);

/*
 * nova_merge_cache_interp with per-image keep counts on the device (see nova_pruned_block_rows):
 *   k           row pitch of kept_idx [B, k] and y_kept [B, k, C]
 *   k_per_row   DEVICE int32 [B] or NULL (= k for every image): only slots [0, k_per_row[b]) of image b are scattered
 *               back (clamped to [0, k]; a slot holding -1 is skipped as well); every other token of the image is
 *               filled from the cache, as keep_mask says.  With k_per_row given, cache_prev is required whatever k is.
 */
int nova_merge_cache_rows(nova_ctx* ctx, void* stream, int dtype, int interp, int B, int C, int h, int w, int hp,
                          int wp, int k, const int32_t* k_per_row, const void* x, const void* y_kept,
                          const int32_t* kept_idx, const uint8_t* keep_mask, const void* cache_prev, void* out,
                          void* cache_new);

/*
 * Ratio controllers (Sec. 3.3, "Adaptive Acceleration Activation" and "Dual-Linkage
 * Acceleration").  The first two are host arithmetic on one instance's scale mean entropies
 * (no GPU work, ctx-free); the third runs on the device so that a layer's keep counts reach
 * nova_select, nova_pruned_block_rows and nova_merge_cache_rows (their k_per_row argument) without a host round trip.
 *
 * nova_activation_scale: with g_t = Hbar_t - Hbar_{t-1}, eta = mean of g_2..g_{t_est} and
 * g~_t = (g_t + g_{t-1}) / 2, *t_star is the earliest t >= t_est + 1 (1-based) with
 * g~_t <= alpha * eta among the scales given, or 0 when there is none (yet); acceleration
 * starts at scale t* + 1.  Appending later scales never changes a detected t*.
 *   hbar   HOST double [T]: Hbar_1 .. Hbar_T; T >= 0, t_est >= 2
 */
int nova_activation_scale(const double* hbar, int T, int t_est, double alpha, int* t_star);

/* Scale-linkage ratio: *ratio = sigmoid((t - (t_star + 1)) / tau) - lambda * tanh(g_t)
 * (host scalars; tau != 0).  Not clamped. */
int nova_scale_ratio(int t, int t_star, double g_t, double tau, double lambda, double* ratio);

/*
 * Layer-linkage ratio and keep counts of layer j (1-based) for every batch row, in fp32:
 *   mu        = entropy_sum[b] / (j - 1)                       (j >= 2)
 *   ratio_tj  = ratio_t[b] - ((mean_entropy[b] - mu) / mu) * ratio_t[b]
 *               (= ratio_t[b] when j == 1 or mu == 0)
 *   k_per_row = N - floor(clamp(ratio_tj, 0, 1) * N)           (a NaN ratio keeps all N)
 *   entropy_sum[b] <- (j == 1 ? 0 : entropy_sum[b]) + mean_entropy[b]
 *   mean_entropy  DEVICE fp32 [B]  this layer's scale mean entropy (nova_entropy's mean output)
 *   entropy_sum   DEVICE fp32 [B]  in/out: sum over the preceding layers of this scale
 *   ratio_t       DEVICE fp32 [B]  scale-linkage ratio of each row
 *   ratio_tj      out DEVICE fp32 [B], not clamped; k_per_row out DEVICE int32 [B]
 * 0 <= N <= 2^24.  B == 0 is a no-op.
 */
int nova_layer_ratio(nova_ctx* ctx, void* stream, const float* mean_entropy, float* entropy_sum,
                     const float* ratio_t, int j, int B, int N, float* ratio_tj, int32_t* k_per_row);

/*
 * Instrumentation (not part of the hot path): per-kernel device timing with HIP events on
 * the caller's stream.  While a stage's bit is set in `stage_mask`, every launch of that
 * stage by the four entry points is bracketed by a pair of events (created on the host as
 * needed).  nova_profile_collect waits for all recorded events, returns the summed elapsed
 * milliseconds and the launch count of `stage` (host pointers, either may be NULL) and
 * releases that stage's events.  A mask of 0 switches timing off (the default).
 */
enum {
  NOVA_STAGE_ENTROPY = 0,   /* nova_entropy kernel                                  */
  NOVA_STAGE_SELECT = 1,    /* nova_select kernel                                   */
  NOVA_STAGE_GATHER_LN = 2, /* nova_pruned_block: gather kept rows + LayerNorm      */
  NOVA_STAGE_QKV = 3,       /*   QKV projection (+ cache append)                    */
  NOVA_STAGE_ATTENTION = 4, /*   attention over prior + kept keys                   */
  NOVA_STAGE_OPROJ = 5,     /*   output projection + residual                       */
  NOVA_STAGE_LN2 = 6,       /*   second LayerNorm                                   */
  NOVA_STAGE_FFN1 = 7,      /*   FFN up projection + GELU                           */
  NOVA_STAGE_FFN2 = 8,      /*   FFN down projection + residual                     */
  NOVA_STAGE_MERGE = 9,     /* nova_merge_cache kernel                              */
  NOVA_STAGE_COUNT = 10
};
int nova_profile_stages(nova_ctx* ctx, uint32_t stage_mask);
int nova_profile_collect(nova_ctx* ctx, int stage, double* total_ms, int64_t* launches);

/*
 * Instrumentation (not part of the hot path): launches one plain kernel that shows what the
 * device sustains, for reading roofline fractions against an achievable figure.  The caller
 * times the launch with events on `stream`; *work (host) receives the bytes moved or the flops
 * done by the launch.
 *   NOVA_PROBE_READ   streams `bytes` from src (16 bytes per lane, grid-stride)
 *   NOVA_PROBE_COPY   copies `bytes` from src to dst (work = 2 * bytes)
 *   NOVA_PROBE_MFMA   8 waves per CU, `iters` rounds of 32 independent bf16 32x32x16 MFMAs each, constant operands
 *   NOVA_PROBE_MFMA_DATA  the same loop on operands read once from src (at least CUs x 512 x 128 bytes of bf16
 *                     values): what the matrix cores sustain depends on the data they are fed
 * src / dst: device, 16-byte aligned; sink: device fp32 [1] (never written in practice).
 */
enum { NOVA_PROBE_READ = 0, NOVA_PROBE_COPY = 1, NOVA_PROBE_MFMA = 2, NOVA_PROBE_MFMA_DATA = 3 };
int nova_probe(nova_ctx* ctx, void* stream, int kind, const void* src, void* dst, int64_t bytes,
               int iters, float* sink, double* work);


#ifdef __cplusplus
}
#endif
#endif /* NOVA_H */
