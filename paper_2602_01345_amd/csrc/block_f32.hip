// fp32 path of the pruned block (Sec. 3.3, "Residual Cache Reuse", first equation,
// evaluated on the kept rows): plain, LDS-tiled fp32 kernels for small fp32 models.
// It exists for correctness at full fp32 precision; the matrix-core path is block_bf16.hip.
#include "common.h"
#include "epilogue.h"
#include "nova_internal.h"

namespace {

constexpr int kTile = 16;

// out[m][n] = sum_k A[m][k] * W[n][k]  (+ epilogue); A [M, K] row-major, W [Nout, K] row-major
template <int MODE>
__global__ __launch_bounds__(kTile* kTile) void gemm_f32_kernel(const float* __restrict__ A,
                                                                const float* __restrict__ W, int M, int Nout,
                                                                int K, EpiParams<float> ep) {
  __shared__ float As[kTile][kTile + 1];
  __shared__ float Ws[kTile][kTile + 1];
  const int tx = threadIdx.x % kTile, ty = threadIdx.x / kTile;
  const int row = blockIdx.y * kTile + ty;
  const int col = blockIdx.x * kTile + tx;
  float acc = 0.f;
  for (int k0 = 0; k0 < K; k0 += kTile) {
    const int ar = blockIdx.y * kTile + ty, wr = blockIdx.x * kTile + ty, kk = k0 + tx;
    As[ty][tx] = (ar < M && kk < K) ? A[(int64_t)ar * K + kk] : 0.f;
    Ws[ty][tx] = (wr < Nout && kk < K) ? W[(int64_t)wr * K + kk] : 0.f;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kTile; ++i) acc = fmaf(As[ty][i], Ws[tx][i], acc);
    __syncthreads();
  }
  if (row < M && col < Nout) epilogue_store<float, MODE>(ep, row, col, acc);
}

// One wave per (query row m, head).  Scores of all P+k cached keys are kept in LDS.
__global__ __launch_bounds__(NOVA_WAVE) void attention_f32_kernel(const float* __restrict__ q,
                                                                  const float* __restrict__ kc,
                                                                  const float* __restrict__ vc, int k, int C,
                                                                  int heads, int dh, int cap, int kv_total_uniform,
                                                                  float scale, float* __restrict__ out,
                                                                  const int32_t* __restrict__ k_rows,
                                                                  const int32_t* __restrict__ kv_rows, int P,
                                                                  int self_keys) {
  extern __shared__ float sc[];            // [kv_total] scores, then [dh] the query
  const int lane = threadIdx.x;
  const int m = blockIdx.x, head = blockIdx.y;
  const int b = m / k;
  // per-image keep counts: a slot past its image's count gets zeros; an image's keys are its own prior rows plus
  // its own kept rows (never more than the uniform total the LDS was sized for)
  const int kq = image_count(k_rows, b, k);
  if (m - b * k >= kq) {
    for (int d = lane; d < dh; d += NOVA_WAVE) out[(int64_t)m * C + head * dh + d] = 0.0f;
    return;
  }
  const int kv_total = self_keys && (k_rows || kv_rows) ? image_prior(kv_rows, b, P) + kq : kv_total_uniform;
  float* qs = sc + kv_total;
  const int64_t bh = (int64_t)b * heads + head;
  const float* K = kc + bh * cap * dh;
  const float* V = vc + bh * dh * (int64_t)cap;
  for (int d = lane; d < dh; d += NOVA_WAVE) qs[d] = q[(int64_t)m * C + head * dh + d];
  __syncthreads();
  float mx = -INFINITY;
  for (int j = lane; j < kv_total; j += NOVA_WAVE) {
    float s = 0.f;
    for (int d = 0; d < dh; ++d) s = fmaf(qs[d], K[(int64_t)j * dh + d], s);
    s *= scale;
    sc[j] = s;
    mx = fmaxf(mx, s);
  }
  mx = wave_max(mx);
  float z = 0.f;
  for (int j = lane; j < kv_total; j += NOVA_WAVE) {
    float e = expf(sc[j] - mx);
    sc[j] = e;
    z += e;
  }
  z = wave_sum(z);
  __syncthreads();
  for (int d = 0; d < dh; ++d) {
    float a = 0.f;
    for (int j = lane; j < kv_total; j += NOVA_WAVE) a = fmaf(sc[j], V[(int64_t)d * cap + j], a);
    a = wave_sum(a);
    if (lane == 0) out[(int64_t)m * C + head * dh + d] = a / z;
  }
}

template <int MODE>
void gemm(hipStream_t st, const float* A, const float* W, int M, int Nout, int K, const EpiParams<float>& ep) {
  dim3 grid((Nout + kTile - 1) / kTile, (M + kTile - 1) / kTile);
  gemm_f32_kernel<MODE><<<grid, kTile * kTile, 0, st>>>(A, W, M, Nout, K, ep);
}

}  // namespace

hipError_t launch_block_f32(nova_ctx* ctx, hipStream_t st, const nova_block_shape& s, const nova_block_weights& w,
                            const nova_block_variant& var, const RowCounts& rc, const float* x, const int32_t* idx,
                            float* kc, float* vc, float* y, const BlockWorkspace& ws) {
  const int M = s.B * s.k, C = s.C, F = s.C * s.ffn_mult, dh = s.C / s.heads;
  float* u = reinterpret_cast<float*>(ws.u);
  float* q = reinterpret_cast<float*>(ws.q);
  float* attn = reinterpret_cast<float*>(ws.attn);
  float* x1 = reinterpret_cast<float*>(ws.x1);
  float* hid = reinterpret_cast<float*>(ws.hid);

  // per-image conditioning vectors [B, 6, C]: shift1, scale1, gate1, shift2, scale2, gate2
  const float* ada = static_cast<const float*>(var.ada);
  const int ada_pitch = 6 * C;
  auto ada_row = [&](int j) { return ada ? ada + (int64_t)j * C : nullptr; };

  hipError_t e;
  {
    StageTimer t(ctx, st, NOVA_STAGE_GATHER_LN);
    e = launch_gather_ln(st, NOVA_F32, x, idx, M, s.k, s.N, C, ada_row(0), ada_row(1), ada_pitch, u, rc.k_rows);
  }
  if (e != hipSuccess) return e;

  EpiParams<float> ep = {};
  ep.C = C; ep.heads = s.heads; ep.dh = dh; ep.cap = s.kv_capacity; ep.P = s.kv_len; ep.k = s.k;
  ep.k_rows = rc.k_rows; ep.kv_rows = rc.kv_rows;
  ep.idx = idx; ep.Ntok = s.N;
  ep.gate_pitch = ada_pitch;

  ep.bias = static_cast<const float*>(w.b_qkv); ep.out = q; ep.ldo = C; ep.kc = kc; ep.vc = vc;
  {
    StageTimer t(ctx, st, NOVA_STAGE_QKV);
    gemm<EPI_QKV>(st, u, static_cast<const float*>(w.w_qkv), M, 3 * C, C, ep);
    if (var.qk_norm) {
      e = launch_qk_norm(st, NOVA_F32, q, kc, var.qk_scale, 1.0f, s.B, s.k, C, s.heads, s.kv_capacity, s.kv_len,
                         rc.k_rows, rc.kv_rows);
      if (e != hipSuccess) return e;
    }
  }

  const int kv_total = s.kv_len + s.k;
  const size_t lds = (size_t)(kv_total + dh) * sizeof(float);
  {
    StageTimer t(ctx, st, NOVA_STAGE_ATTENTION);
    attention_f32_kernel<<<dim3(M, s.heads), NOVA_WAVE, lds, st>>>(q, kc, vc, s.k, C, s.heads, dh, s.kv_capacity,
                                                                   kv_total, var.qk_norm ? 1.0f : 1.0f / sqrtf((float)dh), attn,
                                                                   rc.k_rows, rc.kv_rows, s.kv_len, 1);
  }

  ep.bias = static_cast<const float*>(w.b_o); ep.out = x1; ep.ldo = C; ep.res = x; ep.gate = ada_row(2);
  {
    StageTimer t(ctx, st, NOVA_STAGE_OPROJ);
    gemm<EPI_ATTN_OUT>(st, attn, static_cast<const float*>(w.w_o), M, C, C, ep);
  }
  if (var.w_cq) {
    // cross-attention sub-layer over the condition tokens (see block_bf16.hip)
    e = launch_gather_ln(st, NOVA_F32, x1, nullptr, M, s.k, s.N, C, nullptr, nullptr, 0, u, rc.k_rows);
    if (e != hipSuccess) return e;
    ep.bias = static_cast<const float*>(var.b_cq); ep.out = q; ep.ldo = C; ep.gate = nullptr;
    gemm<EPI_PLAIN>(st, u, static_cast<const float*>(var.w_cq), M, C, C, ep);
    const size_t lds_t = (size_t)(var.text_len + dh) * sizeof(float);
    attention_f32_kernel<<<dim3(M, s.heads), NOVA_WAVE, lds_t, st>>>(
        q, static_cast<const float*>(var.k_text), static_cast<const float*>(var.v_text), s.k, C, s.heads, dh,
        var.text_capacity, var.text_len, 1.0f / sqrtf((float)dh), attn, rc.k_rows, nullptr, 0, 0);
    ep.bias = static_cast<const float*>(var.b_co); ep.out = x1; ep.ldo = C; ep.res = x1;
    gemm<EPI_RESIDUAL>(st, attn, static_cast<const float*>(var.w_co), M, C, C, ep);
  }
  {
    StageTimer t(ctx, st, NOVA_STAGE_LN2);
    e = launch_gather_ln(st, NOVA_F32, x1, nullptr, M, s.k, s.N, C, ada_row(3), ada_row(4), ada_pitch, u, rc.k_rows,
                         rc.kv_rows, rc.kv_next, s.kv_len);
  }
  if (e != hipSuccess) return e;

  ep.bias = static_cast<const float*>(w.b_fc1); ep.out = hid; ep.ldo = F; ep.gate = nullptr;
  {
    StageTimer t(ctx, st, NOVA_STAGE_FFN1);
    if (var.gelu_tanh) gemm<EPI_GELU_TANH>(st, u, static_cast<const float*>(w.w_fc1), M, F, C, ep);
    else gemm<EPI_GELU>(st, u, static_cast<const float*>(w.w_fc1), M, F, C, ep);
  }

  ep.bias = static_cast<const float*>(w.b_fc2); ep.out = y; ep.ldo = C; ep.res = x1; ep.gate = ada_row(5);
  {
    StageTimer t(ctx, st, NOVA_STAGE_FFN2);
    gemm<EPI_RESIDUAL>(st, hid, static_cast<const float*>(w.w_fc2), M, C, F, ep);
  }
  return hipGetLastError();
}
