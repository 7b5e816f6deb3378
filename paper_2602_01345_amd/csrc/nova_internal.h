// Host-side declarations shared by the C ABI (api.hip) and the kernel files.
// Every launch_* function validates nothing: api.hip has already checked the
// arguments against what the kernels and their grids assume.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/nova.h"

#include <vector>

struct ProfRecord {
  int stage;
  hipEvent_t start, stop;
};

struct nova_ctx {
  int device;
  int num_cus;
  size_t lds_per_block;
  uint32_t prof_mask;
  std::vector<ProfRecord> prof;
  int gemm_cfg;   // >= 0 forces one GEMM tile configuration (environment NOVA_GEMM_CFG, for tuning)
  int attn_cfg;   // likewise for the attention kernel (NOVA_ATTN_CFG)
  int attn_split; // >= 1 forces the number of attention key splits (NOVA_ATTN_SPLIT)
  int gemm_parts; // 0 forbids splitting a GEMM's rows over two launches (NOVA_GEMM_PARTS)
  int gemm_persist; // 0: one workgroup per tile always (NOVA_GEMM_PERSIST); else one workgroup per CU walks several tiles
  int gemm_ksplit;  // 0: never cut K of the large-tile FFN down projection into slices; 2 / 4: always (NOVA_GEMM_KSPLIT)
};

// Brackets one kernel launch with a pair of events when its stage is being timed.
struct StageTimer {
  nova_ctx* ctx;
  hipStream_t st;
  hipEvent_t stop;
  bool on;
  StageTimer(nova_ctx* c, hipStream_t s, int stage) : ctx(c), st(s), stop(nullptr), on(false) {
    if (!c || !((c->prof_mask >> stage) & 1u)) return;
    hipEvent_t a = nullptr, b = nullptr;
    if (hipEventCreate(&a) != hipSuccess) return;
    if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return; }
    (void)hipEventRecord(a, s);
    c->prof.push_back({stage, a, b});
    stop = b;
    on = true;
  }
  ~StageTimer() {
    if (on) (void)hipEventRecord(stop, st);
  }
};

// entropy.hip
hipError_t launch_entropy(hipStream_t st, int num_cus, const void* logits, int dtype, int64_t rows_per_batch,
                          int batch, int V, int64_t stride, float* H, float* mean);
// entropy.hip: mean[b] = mean of H[b, 0..rows_per_batch), summed in a fixed order (bit-reproducible)
hipError_t launch_row_mean(hipStream_t st, const float* H, int64_t rows_per_batch, int batch, float* mean);
// select.hip
hipError_t launch_layer_ratio(hipStream_t st, const float* mean_entropy, float* entropy_sum, const float* ratio_t,
                              int j, int B, int N, float* ratio_tj, int32_t* k_per_row);
hipError_t launch_probe_read(hipStream_t st, int num_cus, const void* src, int64_t bytes, float* sink);
hipError_t launch_probe_copy(hipStream_t st, int num_cus, const void* src, void* dst, int64_t bytes);
hipError_t launch_probe_mfma(hipStream_t st, int num_cus, int iters, float* sink);
hipError_t launch_probe_mfma_data(hipStream_t st, int num_cus, const void* src, int iters, float* sink);
hipError_t launch_entropy_bits(hipStream_t st, const void* logits, int dtype, int64_t rows_per_batch, int batch,
                               int d, float* H, float* mean);
hipError_t launch_select(hipStream_t st, const float* H, int B, int N, int k, const int32_t* k_per_row,
                         int32_t* idx, uint8_t* mask);
// merge.hip
hipError_t launch_merge(hipStream_t st, int dtype, int interp, int B, int C, int h, int w, int hp, int wp, int k,
                        const void* x, const void* y, const int32_t* idx, const uint8_t* mask,
                        const void* cache_prev, void* out, void* cache_new, const int32_t* k_rows = nullptr);

// Workspace carving for the block (element counts; every region 256-byte aligned).
struct BlockWorkspace {
  char* u;     // [M, C]  LayerNorm output (reused for both norms)
  char* q;     // [M, C]  queries
  char* attn;  // [M, C]  attention output
  char* x1;    // [M, C]  residual stream after attention
  char* hid;   // [M, F]  FFN hidden
  char* part_o;   // bf16 path: attention partial sums, fp32: max_split per item, [query block][dh] each
  char* part_ml;  // bf16 path: their softmax reference point (log2 units) and sum per query
  int64_t part_floats;   // capacity of part_o in floats (part_ml holds 2 floats per dh of them)
  size_t total;
};
BlockWorkspace carve_workspace(const nova_block_shape& s, void* base);

// norm.hip: dst[m] = LayerNorm(src[row(m)]); with idx, row(m) = (m / k) * N + idx[m], else row(m) = m
// shift / scale: per-image modulation vectors (image = m / k, row pitch mod_pitch elements), both or neither
// k_rows: per-image keep counts (device) or nullptr; slots past an image's count get zero rows.  kv_next (with
// kv_rows, P): the launch also writes the per-image cache lengths after this block, prior rows + kept rows.
hipError_t launch_gather_ln(hipStream_t st, int dtype, const void* src, const int32_t* idx, int M, int k,
                            int N, int C, const void* shift, const void* scale, int mod_pitch, void* dst,
                            const int32_t* k_rows = nullptr, const int32_t* kv_rows = nullptr,
                            int32_t* kv_next = nullptr, int P = 0);
// qk_norm.hip: queries [B*k, C] and the cache's key rows [P, P+k) scaled to unit length per head, in place;
// the queries are also multiplied by qk_scale[head]
hipError_t launch_qk_norm(hipStream_t st, int dtype, void* q, void* kc, const float* qk_scale, float q_mult, int B, int k, int C,
                          int heads, int cap, int P, const int32_t* k_rows = nullptr, const int32_t* kv_rows = nullptr);

// Per-image counts of one block call (device arrays of B entries, or nullptr = uniform): kept tokens per image
// (clamped to [0, shape.k], shape.k being the row pitch), prior K/V rows per image (clamped to [0, shape.kv_len]),
// and where to write the per-image cache lengths after the block (may be the kv_rows array itself).
struct RowCounts {
  const int32_t* k_rows;
  const int32_t* kv_rows;
  int32_t* kv_next;
};

// block_f32.hip: plain fp32 kernels (correctness path for small fp32 models)
hipError_t launch_block_f32(nova_ctx* ctx, hipStream_t st, const nova_block_shape& s, const nova_block_weights& w,
                            const nova_block_variant& var, const RowCounts& rc, const float* x, const int32_t* idx,
                            float* kc, float* vc, float* y, const BlockWorkspace& ws);
// gemm_bf16.hip: out = epilogue(A W^T) on the matrix cores; mode is an EpiMode
template <typename T> struct EpiParams;
hipError_t launch_gemm_bf16(const nova_ctx* ctx, hipStream_t st, int mode, const void* A, const void* W, int M,
                            int Nout, int K, const EpiParams<__bf16>& ep);
int gemm_bf16_tile_cols(const nova_ctx* ctx, int M, int Nout, int K);
size_t head_entropy_workspace_bytes(int M, int V);
hipError_t launch_head_entropy(const nova_ctx* ctx, hipStream_t st, const void* hidden, const void* w_head,
                               const void* b_head, int rows_per_batch, int batch, int C, int V, float* H,
                               float* mean, void* workspace);
// the allocation-free variant's scratch: a static device array in head_entropy.hip.  _init resolves its address
// on `device` once (hipGetSymbolAddress with that device current); _scratch returns it (nullptr before _init)
hipError_t head_entropy_static_init(int device);
void* head_entropy_static_scratch(int device);
size_t head_entropy_static_capacity();
size_t head_entropy_partial_bytes(const nova_ctx* ctx, int M, int V, int C);
// attention_bf16.hip: attn[B*k, C] = softmax(ln 2 * q K^T) V per head over kv_total cached keys: the query rows
// arrive multiplied by (score scale * log2 e) -- kAttnLog2e times the scale of the scores -- by whoever wrote
// them (the projection's epilogue or the unit-length rescaling), so the kernel's scores are in log2 units
// part_o / part_ml: workspace for split-key partial results (part_floats floats, and 2 floats per dh of them),
// or nullptr to forbid splitting
int attention_max_split();
constexpr int kAttentionMaxPieces = 512;      // key runs of cut attention items per launch the workspace has room for
constexpr float kAttnLog2e = 1.4426950408889634f;
// k_rows / kv_rows (device, or nullptr): per-image keep counts and prior-row counts.  Image b's live queries are
// slots [0, k_rows[b]) of its k-slot segment (the other slots get zeros); with self_keys its keys are its own
// kv_rows[b] (default P) prior rows plus its own kept rows, otherwise kv_total keys for every image.
hipError_t launch_attention_bf16(const nova_ctx* ctx, hipStream_t st, const void* q, const void* kc, const void* vc,
                                 int B, int k, int C, int heads, int cap, int kv_total, void* out,
                                 float* part_o, float* part_ml, int64_t part_floats, const int32_t* k_rows = nullptr,
                                 const int32_t* kv_rows = nullptr, int P = 0, int self_keys = 1);
// block_bf16.hip: MFMA path
hipError_t launch_block_bf16(nova_ctx* ctx, hipStream_t st, const nova_block_shape& s,
                             const nova_block_weights& w, const nova_block_variant& var, const RowCounts& rc,
                             const void* x, const int32_t* idx, void* kc, void* vc, void* y,
                             const BlockWorkspace& ws);
