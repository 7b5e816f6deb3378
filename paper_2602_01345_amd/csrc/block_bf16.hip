// bf16 matrix-core path of the pruned block (Sec. 3.3, "Residual Cache Reuse", first
// equation, evaluated on the kept rows only; Sec. 3.2: attention is the cost pruning saves).
//
//   gather+LN -> QKV GEMM (epilogue appends K/V to the caches) -> flash-style attention
//   -> O-proj GEMM (+ residual) -> LN -> FFN1 GEMM (+GELU) -> FFN2 GEMM (+ residual)
//
// Block variants (the backbones of Sec. 4): both norms modulated and both branches gated by per-image
// vectors, queries and keys rescaled to unit length after the QKV GEMM, tanh-form GELU.
//
// The GEMMs live in gemm_bf16.hip, the attention kernel in attention_bf16.hip; this file only
// sequences them on the caller's stream.
#include "common.h"
#include "epilogue.h"
#include "nova_internal.h"

hipError_t launch_block_bf16(nova_ctx* ctx, hipStream_t st, const nova_block_shape& s,
                             const nova_block_weights& w, const nova_block_variant& var, const RowCounts& rc,
                             const void* xv, const int32_t* idx, void* kcv, void* vcv, void* yv,
                             const BlockWorkspace& ws) {
  const int M = s.B * s.k, C = s.C, F = s.C * s.ffn_mult, dh = s.C / s.heads;
  const bf16_t* x = static_cast<const bf16_t*>(xv);
  bf16_t* kc = static_cast<bf16_t*>(kcv);
  bf16_t* vc = static_cast<bf16_t*>(vcv);
  bf16_t* y = static_cast<bf16_t*>(yv);
  bf16_t* u = reinterpret_cast<bf16_t*>(ws.u);
  bf16_t* q = reinterpret_cast<bf16_t*>(ws.q);
  bf16_t* attn = reinterpret_cast<bf16_t*>(ws.attn);
  bf16_t* x1 = reinterpret_cast<bf16_t*>(ws.x1);
  bf16_t* hid = reinterpret_cast<bf16_t*>(ws.hid);

  // per-image conditioning vectors [B, 6, C]: shift1, scale1, gate1, shift2, scale2, gate2
  const bf16_t* ada = static_cast<const bf16_t*>(var.ada);
  const int ada_pitch = 6 * C;
  auto ada_row = [&](int j) { return ada ? ada + (int64_t)j * C : nullptr; };

  hipError_t e;
  {
    StageTimer t(ctx, st, NOVA_STAGE_GATHER_LN);
    e = launch_gather_ln(st, NOVA_BF16, x, idx, M, s.k, s.N, C, ada_row(0), ada_row(1), ada_pitch, u, rc.k_rows);
  }
  if (e != hipSuccess) return e;

  EpiParams<bf16_t> ep = {};
  ep.C = C; ep.heads = s.heads; ep.dh = dh; ep.cap = s.kv_capacity; ep.P = s.kv_len; ep.k = s.k;
  ep.idx = idx; ep.Ntok = s.N;
  ep.k_rows = rc.k_rows; ep.kv_rows = rc.kv_rows;
  ep.gate_pitch = ada_pitch;
  ep.part = reinterpret_cast<float*>(ws.part_o);          // free once attention is done: K-slice sums of the projections back to C
  ep.part_floats = ws.part_floats;

  // the attention kernel takes its query rows multiplied by (score scale * log2 e); unit-length queries get the
  // factor when they are rescaled (a factor before that would cancel)
  ep.bias = static_cast<const bf16_t*>(w.b_qkv); ep.out = q; ep.ldo = C; ep.kc = kc; ep.vc = vc;
  ep.q_scale = var.qk_norm ? 1.0f : kAttnLog2e / sqrtf((float)dh);
  {
    StageTimer t(ctx, st, NOVA_STAGE_QKV);
    e = launch_gemm_bf16(ctx, st, EPI_QKV, u, w.w_qkv, M, 3 * C, C, ep);
    if (e == hipSuccess && var.qk_norm)
      e = launch_qk_norm(st, NOVA_BF16, q, kc, var.qk_scale, kAttnLog2e, s.B, s.k, C, s.heads, s.kv_capacity, s.kv_len,
                         rc.k_rows, rc.kv_rows);
  }
  if (e != hipSuccess) return e;

  {
    StageTimer t(ctx, st, NOVA_STAGE_ATTENTION);
    e = launch_attention_bf16(ctx, st, q, kc, vc, s.B, s.k, C, s.heads, s.kv_capacity, s.kv_len + s.k, attn,
                              reinterpret_cast<float*>(ws.part_o), reinterpret_cast<float*>(ws.part_ml), ws.part_floats,
                              rc.k_rows, rc.kv_rows, s.kv_len, 1);
  }
  if (e != hipSuccess) return e;

  ep.bias = static_cast<const bf16_t*>(w.b_o); ep.out = x1; ep.ldo = C; ep.res = x; ep.gate = ada_row(2);
  {
    StageTimer t(ctx, st, NOVA_STAGE_OPROJ);
    e = launch_gemm_bf16(ctx, st, EPI_ATTN_OUT, attn, w.w_o, M, C, C, ep);
  }
  if (e != hipSuccess) return e;
  if (var.w_cq) {
    // cross-attention sub-layer over the condition tokens: LN -> query projection -> attention over the
    // text keys / values -> output projection added to x1 in place (each output element is read and
    // written by the same thread)
    e = launch_gather_ln(st, NOVA_BF16, x1, nullptr, M, s.k, s.N, C, nullptr, nullptr, 0, u, rc.k_rows);
    if (e != hipSuccess) return e;
    ep.bias = static_cast<const bf16_t*>(var.b_cq); ep.out = q; ep.ldo = C; ep.gate = nullptr;
    ep.q_scale = kAttnLog2e / sqrtf((float)dh);
    e = launch_gemm_bf16(ctx, st, EPI_PLAIN, u, var.w_cq, M, C, C, ep);
    if (e != hipSuccess) return e;
    e = launch_attention_bf16(ctx, st, q, var.k_text, var.v_text, s.B, s.k, C, s.heads, var.text_capacity,
                              var.text_len, attn, reinterpret_cast<float*>(ws.part_o),
                              reinterpret_cast<float*>(ws.part_ml), ws.part_floats, rc.k_rows, nullptr, 0, 0);
    if (e != hipSuccess) return e;
    ep.bias = static_cast<const bf16_t*>(var.b_co); ep.out = x1; ep.ldo = C; ep.res = x1;
    e = launch_gemm_bf16(ctx, st, EPI_RESIDUAL, attn, var.w_co, M, C, C, ep);
    if (e != hipSuccess) return e;
  }
  {
    StageTimer t(ctx, st, NOVA_STAGE_LN2);
    e = launch_gather_ln(st, NOVA_BF16, x1, nullptr, M, s.k, s.N, C, ada_row(3), ada_row(4), ada_pitch, u, rc.k_rows,
                         rc.kv_rows, rc.kv_next, s.kv_len);
  }
  if (e != hipSuccess) return e;

  ep.bias = static_cast<const bf16_t*>(w.b_fc1); ep.out = hid; ep.ldo = F; ep.gate = nullptr;
  {
    StageTimer t(ctx, st, NOVA_STAGE_FFN1);
    e = launch_gemm_bf16(ctx, st, var.gelu_tanh ? EPI_GELU_TANH : EPI_GELU, u, w.w_fc1, M, F, C, ep);
  }
  if (e != hipSuccess) return e;

  ep.bias = static_cast<const bf16_t*>(w.b_fc2); ep.out = y; ep.ldo = C; ep.res = x1; ep.gate = ada_row(5);
  {
    StageTimer t(ctx, st, NOVA_STAGE_FFN2);
    e = launch_gemm_bf16(ctx, st, EPI_RESIDUAL, hid, w.w_fc2, M, C, F, ep);
  }
  return hipGetLastError();
}
