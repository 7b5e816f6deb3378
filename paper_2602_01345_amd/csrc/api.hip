// C ABI of the library (declared in include/nova.h): argument checks on the host,
// then dispatch to the kernel launchers.  No allocation, no synchronisation.
#include <algorithm>
#include <cstdlib>
#include <new>

#include "nova_internal.h"

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
inline size_t esize(int dtype) { return dtype == NOVA_BF16 ? 2 : 4; }
inline bool valid_dtype(int dtype) { return dtype == NOVA_F32 || dtype == NOVA_BF16; }
inline size_t up256(size_t v) { return (v + 255) & ~size_t(255); }

int shape_error(const nova_block_shape* s) {
  if (!s) return NOVA_ERR_INVALID_ARG;
  if (!valid_dtype(s->dtype)) return NOVA_ERR_UNSUPPORTED;
  if (s->B < 0 || s->N < 0 || s->C < 1 || s->heads < 1 || s->ffn_mult < 1 || s->kv_len < 0 || s->k < 0)
    return NOVA_ERR_INVALID_ARG;
  if (s->k > s->N) return NOVA_ERR_INVALID_ARG;
  if (s->C % s->heads != 0) return NOVA_ERR_INVALID_ARG;
  if ((int64_t)s->kv_len + s->k > s->kv_capacity) return NOVA_ERR_INVALID_ARG;
  const int dh = s->C / s->heads;
  if (s->dtype == NOVA_BF16) {
    if (s->C % 64 != 0 || (dh != 64 && dh != 128) || s->kv_capacity % 64 != 0) return NOVA_ERR_UNSUPPORTED;
  } else {
    if (s->C % 4 != 0 || dh > 256) return NOVA_ERR_UNSUPPORTED;
    // the fp32 attention keeps one score per cached key (plus the query) in 64 KiB of LDS
    if ((int64_t)s->kv_len + s->k + dh > 16384) return NOVA_ERR_UNSUPPORTED;
  }
  if ((int64_t)s->B * s->k * (int64_t)s->C * s->ffn_mult > (int64_t)1 << 40) return NOVA_ERR_UNSUPPORTED;
  return NOVA_OK;
}

int set_device(const nova_ctx* ctx) {
  int cur = -1;
  if (hipGetDevice(&cur) != hipSuccess) return NOVA_ERR_HIP;
  if (cur != ctx->device && hipSetDevice(ctx->device) != hipSuccess) return NOVA_ERR_HIP;
  return NOVA_OK;
}

}  // namespace

BlockWorkspace carve_workspace(const nova_block_shape& s, void* base) {
  const size_t M = (size_t)s.B * s.k, C = s.C, F = (size_t)s.C * s.ffn_mult, e = esize(s.dtype);
  BlockWorkspace w;
  char* p = static_cast<char*>(base);
  size_t off = 0;
  w.u = p + off;    off += up256(M * C * e);
  w.q = p + off;    off += up256(M * C * e);
  w.attn = p + off; off += up256(M * C * e);
  w.x1 = p + off;   off += up256(M * C * e);
  w.hid = p + off;  off += up256(M * F * e);
  w.part_o = w.part_ml = nullptr;
  w.part_floats = 0;
  if (s.dtype == NOVA_BF16) {
    // One region serves two users, one after the other: the partial results of the attention items that are cut
    // into key runs (only the items of the last, partly filled round over the workgroup slots are: at most
    // kAttentionMaxPieces runs of up to 256 queries x dh floats, or attention_max_split() per item when the call
    // is small), and the fp32 K-slice sums of the projections back to C (slices x rows x C for launches whose tiles
    // fill at most half of the compute units: at most 128 tiles of 256 x 256).
    const size_t dh = (size_t)(s.C / s.heads);
    const size_t Mp = (size_t)s.B * (((size_t)s.k + 255) / 256 * 256);
    const size_t attn = std::min((size_t)attention_max_split() * Mp * C, (size_t)kAttentionMaxPieces * 256 * dh);
    const size_t kslice = std::min((size_t)4 * M * C, (size_t)128 * 256 * 256);
    w.part_floats = (int64_t)std::max(attn, kslice);
    w.part_o = p + off;  off += up256((size_t)w.part_floats * 4);
    w.part_ml = p + off; off += up256((size_t)w.part_floats / dh * 2 * 4);     // (reference, sum) per query and run
  }
  w.total = off;
  return w;
}

extern "C" {

int nova_create(nova_ctx** out, int device_id) {
  if (!out) return NOVA_ERR_INVALID_ARG;
  *out = nullptr;
  int n = 0;
  if (hipGetDeviceCount(&n) != hipSuccess) return NOVA_ERR_HIP;
  if (device_id < 0 || device_id >= n) return NOVA_ERR_INVALID_ARG;
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, device_id) != hipSuccess) return NOVA_ERR_HIP;
  // the allocation-free entry point's scratch is a static device array: resolve its address on this device now
  if (head_entropy_static_init(device_id) != hipSuccess) return NOVA_ERR_HIP;
  nova_ctx* c = new (std::nothrow) nova_ctx;
  if (!c) return NOVA_ERR_HIP;
  c->device = device_id;
  c->num_cus = prop.multiProcessorCount;
  c->lds_per_block = prop.sharedMemPerBlock;
  c->prof_mask = 0;
  const char* g = getenv("NOVA_GEMM_CFG");
  const char* a = getenv("NOVA_ATTN_CFG");
  c->gemm_cfg = g ? atoi(g) : -1;
  c->attn_cfg = a ? atoi(a) : -1;
  const char* sp = getenv("NOVA_ATTN_SPLIT");
  c->attn_split = sp ? atoi(sp) : -1;
  const char* gp = getenv("NOVA_GEMM_PARTS");
  c->gemm_parts = gp ? atoi(gp) : -1;
  const char* gs = getenv("NOVA_GEMM_PERSIST");
  c->gemm_persist = gs ? atoi(gs) : -1;
  const char* gk = getenv("NOVA_GEMM_KSPLIT");
  c->gemm_ksplit = gk ? atoi(gk) : -1;
  *out = c;
  return NOVA_OK;
}

int nova_destroy(nova_ctx* ctx) {
  if (ctx) {
    for (ProfRecord& r : ctx->prof) {
      (void)hipEventDestroy(r.start);
      (void)hipEventDestroy(r.stop);
    }
  }
  delete ctx;
  return NOVA_OK;
}

int nova_probe(nova_ctx* ctx, void* stream, int kind, const void* src, void* dst, int64_t bytes, int iters,
               float* sink, double* work) {
  if (!ctx || !sink || !work) return NOVA_ERR_INVALID_ARG;
  if (int rc = set_device(ctx)) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipError_t e = hipSuccess;
  switch (kind) {
    case NOVA_PROBE_READ:
      if (!src || bytes < 16 || reinterpret_cast<uintptr_t>(src) % 16) return NOVA_ERR_INVALID_ARG;
      e = launch_probe_read(st, ctx->num_cus, src, bytes, sink);
      *work = (double)(bytes / 16 * 16);
      break;
    case NOVA_PROBE_COPY:
      if (!src || !dst || bytes < 16 || reinterpret_cast<uintptr_t>(src) % 16 || reinterpret_cast<uintptr_t>(dst) % 16)
        return NOVA_ERR_INVALID_ARG;
      e = launch_probe_copy(st, ctx->num_cus, src, dst, bytes);
      *work = 2.0 * (double)(bytes / 16 * 16);
      break;
    case NOVA_PROBE_MFMA:
      if (iters < 1) return NOVA_ERR_INVALID_ARG;
      e = launch_probe_mfma(st, ctx->num_cus, iters, sink);
      // workgroups x waves x rounds x MFMAs x flops of one 32x32x16 MFMA
      *work = (double)ctx->num_cus * 8.0 * (double)iters * 32.0 * (2.0 * 32 * 32 * 16);
      break;
    case NOVA_PROBE_MFMA_DATA:
      // every lane reads 128 bytes of operands: num_cus workgroups of 512 lanes
      if (iters < 1 || !src || reinterpret_cast<uintptr_t>(src) % 16 || bytes < (int64_t)ctx->num_cus * 512 * 128)
        return NOVA_ERR_INVALID_ARG;
      e = launch_probe_mfma_data(st, ctx->num_cus, src, iters, sink);
      *work = (double)ctx->num_cus * 8.0 * (double)iters * 32.0 * (2.0 * 32 * 32 * 16);
      break;
    default: return NOVA_ERR_INVALID_ARG;
  }
  return e == hipSuccess ? NOVA_OK : NOVA_ERR_HIP;
}

int nova_profile_stages(nova_ctx* ctx, uint32_t stage_mask) {
  if (!ctx || (stage_mask >> NOVA_STAGE_COUNT) != 0) return NOVA_ERR_INVALID_ARG;
  ctx->prof_mask = stage_mask;
  return NOVA_OK;
}

int nova_profile_collect(nova_ctx* ctx, int stage, double* total_ms, int64_t* launches) {
  if (!ctx || stage < 0 || stage >= NOVA_STAGE_COUNT) return NOVA_ERR_INVALID_ARG;
  double ms = 0.0;
  int64_t n = 0;
  int rc = NOVA_OK;
  std::vector<ProfRecord> keep;
  for (ProfRecord& r : ctx->prof) {
    if (r.stage != stage) { keep.push_back(r); continue; }
    float t = 0.f;
    if (hipEventSynchronize(r.stop) != hipSuccess || hipEventElapsedTime(&t, r.start, r.stop) != hipSuccess)
      rc = NOVA_ERR_HIP;
    else { ms += t; ++n; }
    (void)hipEventDestroy(r.start);
    (void)hipEventDestroy(r.stop);
  }
  ctx->prof.swap(keep);
  if (total_ms) *total_ms = ms;
  if (launches) *launches = n;
  return rc;
}

const char* nova_strerror(int code) {
  switch (code) {
    case NOVA_OK: return "ok";
    case NOVA_ERR_INVALID_ARG: return "invalid argument";
    case NOVA_ERR_UNSUPPORTED: return "unsupported shape or dtype";
    case NOVA_ERR_WORKSPACE: return "workspace too small or misaligned";
    case NOVA_ERR_HIP: return "HIP runtime error";
    case NOVA_ERR_STATIC_SCRATCH: return "request exceeds the static scratch of the allocation-free entry point";
    default: return "unknown error code";
  }
}

size_t nova_workspace_bytes(const nova_block_shape* shape) {
  if (shape_error(shape) != NOVA_OK || shape->k == 0 || shape->B == 0) return 0;
  return carve_workspace(*shape, nullptr).total;
}

int nova_entropy(nova_ctx* ctx, void* stream, const void* logits, int logits_dtype, int64_t rows_per_batch,
                 int batch, int V, int64_t row_stride_elems, float* entropy, float* mean_entropy) {
  if (!ctx) return NOVA_ERR_INVALID_ARG;
  if (!valid_dtype(logits_dtype)) return NOVA_ERR_UNSUPPORTED;
  if (rows_per_batch < 0 || batch < 0 || V < 1 || row_stride_elems < V) return NOVA_ERR_INVALID_ARG;
  if (rows_per_batch == 0 || batch == 0) return NOVA_OK;
  if (!logits || !entropy) return NOVA_ERR_INVALID_ARG;
  if (rows_per_batch * batch > ((int64_t)1 << 31) - 8) return NOVA_ERR_UNSUPPORTED;
  if ((reinterpret_cast<uintptr_t>(logits) % esize(logits_dtype)) != 0) return NOVA_ERR_INVALID_ARG;
  if (int rc = set_device(ctx)) return rc;
  StageTimer timer(ctx, static_cast<hipStream_t>(stream), NOVA_STAGE_ENTROPY);
  hipError_t e = launch_entropy(static_cast<hipStream_t>(stream), ctx->num_cus, logits, logits_dtype, rows_per_batch, batch, V,
                                row_stride_elems, entropy, mean_entropy);
  return e == hipSuccess ? NOVA_OK : NOVA_ERR_HIP;
}

int nova_entropy_bits(nova_ctx* ctx, void* stream, const void* bit_logits, int logits_dtype,
                      int64_t rows_per_batch, int batch, int d, float* entropy, float* mean_entropy) {
  if (!ctx) return NOVA_ERR_INVALID_ARG;
  if (!valid_dtype(logits_dtype)) return NOVA_ERR_UNSUPPORTED;
  if (rows_per_batch < 0 || batch < 0 || d < 1) return NOVA_ERR_INVALID_ARG;
  if (rows_per_batch == 0 || batch == 0) return NOVA_OK;
  if (!bit_logits || !entropy) return NOVA_ERR_INVALID_ARG;
  if (rows_per_batch * batch > ((int64_t)1 << 31) - 8) return NOVA_ERR_UNSUPPORTED;
  if ((reinterpret_cast<uintptr_t>(bit_logits) % esize(logits_dtype)) != 0) return NOVA_ERR_INVALID_ARG;
  if (int rc = set_device(ctx)) return rc;
  hipError_t e = launch_entropy_bits(static_cast<hipStream_t>(stream), bit_logits, logits_dtype, rows_per_batch,
                                     batch, d, entropy, mean_entropy);
  return e == hipSuccess ? NOVA_OK : NOVA_ERR_HIP;
}

size_t nova_head_entropy_workspace_bytes(int64_t rows_per_batch, int batch, int V) {
  if (rows_per_batch <= 0 || batch <= 0 || V < 1 || rows_per_batch * batch > ((int64_t)1 << 24)) return 0;
  return head_entropy_workspace_bytes((int)(rows_per_batch * batch), V);
}

int nova_head_entropy(nova_ctx* ctx, void* stream, const void* hidden, const void* w_head, const void* b_head,
                      int dtype, int64_t rows_per_batch, int batch, int C, int V, float* entropy,
                      float* mean_entropy, void* workspace, size_t workspace_bytes) {
  if (!ctx) return NOVA_ERR_INVALID_ARG;
  if (dtype != NOVA_BF16) return NOVA_ERR_UNSUPPORTED;
  if (rows_per_batch < 0 || batch < 0 || V < 1 || C < 1) return NOVA_ERR_INVALID_ARG;
  if (rows_per_batch == 0 || batch == 0) return NOVA_OK;
  if (rows_per_batch * batch > ((int64_t)1 << 24)) return NOVA_ERR_UNSUPPORTED;
  if (C % 64 != 0) return NOVA_ERR_UNSUPPORTED;
  if (!hidden || !w_head || !entropy || !workspace) return NOVA_ERR_INVALID_ARG;
  for (const void* p : {hidden, w_head, b_head, (const void*)workspace})
    if (reinterpret_cast<uintptr_t>(p) % 16 != 0) return NOVA_ERR_INVALID_ARG;
  if (workspace_bytes < nova_head_entropy_workspace_bytes(rows_per_batch, batch, V)) return NOVA_ERR_WORKSPACE;
  if (int rc = set_device(ctx)) return rc;
  hipError_t e = launch_head_entropy(ctx, static_cast<hipStream_t>(stream), hidden, w_head, b_head,
                                     (int)rows_per_batch, batch, C, V, entropy, mean_entropy, workspace);
  return e == hipSuccess ? NOVA_OK : NOVA_ERR_HIP;
}

int nova_head_entropy_static(nova_ctx* ctx, void* stream, const void* hidden, const void* w_head,
                             const void* b_head, int dtype, int64_t rows_per_batch, int batch, int C, int V,
                             float* entropy, float* mean_entropy) {
  if (!ctx) return NOVA_ERR_INVALID_ARG;
  if (dtype != NOVA_BF16) return NOVA_ERR_UNSUPPORTED;
  if (rows_per_batch < 0 || batch < 0 || V < 1 || C < 1) return NOVA_ERR_INVALID_ARG;
  if (rows_per_batch == 0 || batch == 0) return NOVA_OK;
  if (rows_per_batch * batch > ((int64_t)1 << 24)) return NOVA_ERR_UNSUPPORTED;
  if (C % 64 != 0) return NOVA_ERR_UNSUPPORTED;
  if (!hidden || !w_head || !entropy) return NOVA_ERR_INVALID_ARG;
  for (const void* p : {hidden, w_head, b_head})
    if (reinterpret_cast<uintptr_t>(p) % 16 != 0) return NOVA_ERR_INVALID_ARG;
  if (head_entropy_partial_bytes(ctx, (int)(rows_per_batch * batch), V, C) > head_entropy_static_capacity())
    return NOVA_ERR_STATIC_SCRATCH;
  void* scratch_ptr = head_entropy_static_scratch(ctx->device);     // resolved by nova_create on this device
  if (!scratch_ptr) return NOVA_ERR_HIP;
  if (int rc = set_device(ctx)) return rc;
  hipError_t e = launch_head_entropy(ctx, static_cast<hipStream_t>(stream), hidden, w_head, b_head,
                                     (int)rows_per_batch, batch, C, V, entropy, mean_entropy, scratch_ptr);
  return e == hipSuccess ? NOVA_OK : NOVA_ERR_HIP;
}

int nova_select(nova_ctx* ctx, void* stream, const float* entropy, int B, int N, int k, const int32_t* k_per_row,
                int32_t* kept_idx, uint8_t* keep_mask) {
  if (!ctx) return NOVA_ERR_INVALID_ARG;
  if (B < 0 || N < 0 || k < 0 || k > N) return NOVA_ERR_INVALID_ARG;
  if (N > 65536) return NOVA_ERR_UNSUPPORTED;
  if (B == 0 || N == 0) return NOVA_OK;
  if (!entropy || !keep_mask || (k > 0 && !kept_idx)) return NOVA_ERR_INVALID_ARG;
  if (int rc = set_device(ctx)) return rc;
  StageTimer timer(ctx, static_cast<hipStream_t>(stream), NOVA_STAGE_SELECT);
  hipError_t e = launch_select(static_cast<hipStream_t>(stream), entropy, B, N, k, k_per_row, kept_idx, keep_mask);
  return e == hipSuccess ? NOVA_OK : NOVA_ERR_HIP;
}

int nova_layer_ratio(nova_ctx* ctx, void* stream, const float* mean_entropy, float* entropy_sum,
                     const float* ratio_t, int j, int B, int N, float* ratio_tj, int32_t* k_per_row) {
  if (!ctx) return NOVA_ERR_INVALID_ARG;
  if (j < 1 || B < 0 || N < 0 || N > (1 << 24)) return NOVA_ERR_INVALID_ARG;
  if (B == 0) return NOVA_OK;
  if (!mean_entropy || !entropy_sum || !ratio_t || !ratio_tj || !k_per_row) return NOVA_ERR_INVALID_ARG;
  if (int rc = set_device(ctx)) return rc;
  hipError_t e = launch_layer_ratio(static_cast<hipStream_t>(stream), mean_entropy, entropy_sum, ratio_t, j, B, N,
                                    ratio_tj, k_per_row);
  return e == hipSuccess ? NOVA_OK : NOVA_ERR_HIP;
}

int nova_pruned_block(nova_ctx* ctx, void* stream, const nova_block_shape* shape,
                      const nova_block_weights* weights, const void* x, const int32_t* kept_idx, void* k_cache,
                      void* v_cache, void* y_kept, void* workspace, size_t workspace_bytes) {
  return nova_pruned_block_variant(ctx, stream, shape, weights, nullptr, x, kept_idx, k_cache, v_cache, y_kept,
                                   workspace, workspace_bytes);
}

int nova_pruned_block_variant(nova_ctx* ctx, void* stream, const nova_block_shape* shape,
                              const nova_block_weights* weights, const nova_block_variant* variant,
                              const void* x, const int32_t* kept_idx, void* k_cache, void* v_cache, void* y_kept,
                              void* workspace, size_t workspace_bytes) {
  return nova_pruned_block_rows(ctx, stream, shape, weights, variant, nullptr, nullptr, nullptr, x, kept_idx, k_cache,
                                v_cache, y_kept, workspace, workspace_bytes);
}

int nova_pruned_block_rows(nova_ctx* ctx, void* stream, const nova_block_shape* shape,
                           const nova_block_weights* weights, const nova_block_variant* variant,
                           const int32_t* k_per_row, const int32_t* kv_len_per_row, int32_t* kv_len_next,
                           const void* x, const int32_t* kept_idx, void* k_cache, void* v_cache, void* y_kept,
                           void* workspace, size_t workspace_bytes) {
  if (!ctx || !weights) return NOVA_ERR_INVALID_ARG;
  for (const void* p : {(const void*)k_per_row, (const void*)kv_len_per_row, (const void*)kv_len_next})
    if (reinterpret_cast<uintptr_t>(p) & 3) return NOVA_ERR_INVALID_ARG;
  const RowCounts rows = {k_per_row, kv_len_per_row, kv_len_next};
  nova_block_variant var = {};
  if (variant) var = *variant;
  if ((var.gelu_tanh != 0 && var.gelu_tanh != 1) || (var.qk_norm != 0 && var.qk_norm != 1))
    return NOVA_ERR_INVALID_ARG;
  if (var.qk_norm && (!var.qk_scale || (reinterpret_cast<uintptr_t>(var.qk_scale) & 3) != 0))
    return NOVA_ERR_INVALID_ARG;
  if (var.ada && !aligned16(var.ada)) return NOVA_ERR_INVALID_ARG;
  if (int rc = shape_error(shape)) return rc;
  if (var.w_cq) {
    if (!var.w_co || !var.k_text || !var.v_text) return NOVA_ERR_INVALID_ARG;
    if (var.text_len < 1 || var.text_len > var.text_capacity) return NOVA_ERR_INVALID_ARG;
    const void* cptrs[] = {var.w_cq, var.b_cq, var.w_co, var.b_co, var.k_text, var.v_text};
    for (const void* p : cptrs)
      if (p && !aligned16(p)) return NOVA_ERR_INVALID_ARG;
    const int dh = shape->C / shape->heads;
    if (shape->dtype == NOVA_BF16 ? var.text_capacity % 64 != 0 : (int64_t)var.text_len + dh > 16384)
      return NOVA_ERR_UNSUPPORTED;
  }
  if (shape->k == 0 || shape->B == 0) return NOVA_OK;
  if (!x || !kept_idx || !k_cache || !v_cache || !y_kept) return NOVA_ERR_INVALID_ARG;
  if (!weights->w_qkv || !weights->w_o || !weights->w_fc1 || !weights->w_fc2) return NOVA_ERR_INVALID_ARG;
  const void* ptrs[] = {x, k_cache, v_cache, y_kept, weights->w_qkv, weights->w_o, weights->w_fc1, weights->w_fc2,
                        weights->b_qkv, weights->b_o, weights->b_fc1, weights->b_fc2};
  for (const void* p : ptrs)
    if (p && !aligned16(p)) return NOVA_ERR_INVALID_ARG;
  const size_t need = carve_workspace(*shape, nullptr).total;
  if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0)
    return NOVA_ERR_WORKSPACE;
  if (int rc = set_device(ctx)) return rc;
  const BlockWorkspace ws = carve_workspace(*shape, workspace);
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipError_t e;
  if (shape->dtype == NOVA_BF16)
    e = launch_block_bf16(ctx, st, *shape, *weights, var, rows, x, kept_idx, k_cache, v_cache, y_kept, ws);
  else
    e = launch_block_f32(ctx, st, *shape, *weights, var, rows, static_cast<const float*>(x), kept_idx,
                         static_cast<float*>(k_cache), static_cast<float*>(v_cache), static_cast<float*>(y_kept), ws);
  return e == hipSuccess ? NOVA_OK : NOVA_ERR_HIP;
}

int nova_merge_cache(nova_ctx* ctx, void* stream, int dtype, int B, int C, int h, int w, int hp, int wp, int k,
                     const void* x, const void* y_kept, const int32_t* kept_idx, const uint8_t* keep_mask,
                     const void* cache_prev, void* out, void* cache_new) {
  return nova_merge_cache_interp(ctx, stream, dtype, NOVA_INTERP_BILINEAR, B, C, h, w, hp, wp, k, x, y_kept, kept_idx,
                                 keep_mask, cache_prev, out, cache_new);
}

int nova_merge_cache_interp(nova_ctx* ctx, void* stream, int dtype, int interp, int B, int C, int h, int w, int hp,
                            int wp, int k, const void* x, const void* y_kept, const int32_t* kept_idx,
                            const uint8_t* keep_mask, const void* cache_prev, void* out, void* cache_new) {
  return nova_merge_cache_rows(ctx, stream, dtype, interp, B, C, h, w, hp, wp, k, nullptr, x, y_kept, kept_idx,
                               keep_mask, cache_prev, out, cache_new);
}

int nova_merge_cache_rows(nova_ctx* ctx, void* stream, int dtype, int interp, int B, int C, int h, int w, int hp,
                          int wp, int k, const int32_t* k_per_row, const void* x, const void* y_kept,
                          const int32_t* kept_idx, const uint8_t* keep_mask, const void* cache_prev, void* out,
                          void* cache_new) {
  if (!ctx) return NOVA_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(k_per_row) & 3) return NOVA_ERR_INVALID_ARG;
  if (interp != NOVA_INTERP_BILINEAR && interp != NOVA_INTERP_NEAREST && interp != NOVA_INTERP_BICUBIC)
    return NOVA_ERR_INVALID_ARG;
  if (!valid_dtype(dtype)) return NOVA_ERR_UNSUPPORTED;
  if (B < 0 || C < 1 || h < 0 || w < 0 || k < 0) return NOVA_ERR_INVALID_ARG;
  const int64_t N = (int64_t)h * w;
  if (k > N || N > ((int64_t)1 << 30)) return NOVA_ERR_INVALID_ARG;
  if (B == 0 || N == 0) return NOVA_OK;
  if (C % (16 / (int)esize(dtype)) != 0) return NOVA_ERR_UNSUPPORTED;
  if (!x || !out || !keep_mask || out == x) return NOVA_ERR_INVALID_ARG;
  if (k > 0 && (!y_kept || !kept_idx)) return NOVA_ERR_INVALID_ARG;
  // with per-image counts some image may keep fewer than k tokens: the prior cache is needed whatever k is
  if ((k < N || k_per_row) && (!cache_prev || hp < 1 || wp < 1)) return NOVA_ERR_INVALID_ARG;
  if (hp < 1 || wp < 1) cache_prev = nullptr;   // only reachable with k == N: an empty prior grid is never sampled
  const void* ptrs[] = {x, y_kept, cache_prev, out, cache_new};
  for (const void* p : ptrs)
    if (p && !aligned16(p)) return NOVA_ERR_INVALID_ARG;
  if (int rc = set_device(ctx)) return rc;
  StageTimer timer(ctx, static_cast<hipStream_t>(stream), NOVA_STAGE_MERGE);
  hipError_t e = launch_merge(static_cast<hipStream_t>(stream), dtype, interp, B, C, h, w, hp, wp, k, x, y_kept, kept_idx,
                              keep_mask, cache_prev, out, cache_new, k_per_row);
  return e == hipSuccess ? NOVA_OK : NOVA_ERR_HIP;
}

}  // extern "C"
