// Fused GEMM epilogues of the pruned block: what happens to one fp32 accumulator
// element (row = kept-token row m in [0, B*k), col = output feature) once the
// projection y = u W^T is done.
#pragma once
#include "common.h"

enum EpiMode {
  EPI_QKV = 0,        // + b_qkv; split into q (workspace), key rows and value columns of the caches
  EPI_ATTN_OUT = 1,   // x1 = x[gathered row] + acc + b_o
  EPI_GELU = 2,       // hid = GELU(acc + b_fc1), erf form
  EPI_RESIDUAL = 3,   // y = x1 + acc + b_fc2
  EPI_ENTROPY = 4,    // acc + b are logits: only per-row softmax-entropy partials of the tile's columns leave the kernel
  EPI_GELU_TANH = 5,  // EPI_GELU with the tanh form
  EPI_PLAIN = 6,      // out = acc + b (the query projection of a cross-attention sub-layer)
  EPI_PARTIAL = 7     // raw fp32 sums over one slice of K, [slice][M][Nout]; a reduce pass applies the real epilogue
};

template <typename T>
struct EpiParams {
  const T* bias;        // [Nout] or nullptr
  T* out;               // q | x1 | hid | y, row pitch ldo
  int ldo;
  // EPI_QKV
  T* kc;                // [B, heads, cap, dh]
  T* vc;                // [B, heads, dh, cap]
  int C, heads, dh, cap, P, k;
  // per-image counts (device, or nullptr = uniform): image b keeps rows [0, k_rows[b]) of its k-row segment and
  // appends them behind its own kv_rows[b] prior rows; rows past an image's count are computed but never appended,
  // and output tiles that hold no live row are skipped
  const int32_t* k_rows;
  const int32_t* kv_rows;
  // residual sources
  const T* res;         // EPI_ATTN_OUT: x [B, Ntok, C] gathered through idx; EPI_RESIDUAL: x1 [M, C]
  const int32_t* idx;   // [B, k]
  int Ntok;
  // block variants: per-image gate on the projection before the residual is added (EPI_ATTN_OUT, EPI_RESIDUAL),
  // gate[(row / k) * gate_pitch + col], nullptr = 1
  const T* gate;
  int gate_pitch;
  // EPI_ENTROPY: [column tiles][M] partials (m, S, T, unused) with S = sum e^(x-m), T = sum (m-x) e^(x-m)
  f32x4* ent_part;
  // bf16 kernels: factor on the query features (EPI_QKV: columns < C; EPI_PLAIN: all) before they are rounded --
  // the attention kernel wants its queries multiplied by (score scale * log2 e)
  float q_scale;
  // K slicing (few rows, long K): fp32 scratch for [slices][rows of the launch][Nout] partial sums (part_floats
  // floats), or nullptr to forbid slicing
  float* part;
  int64_t part_floats;
};

// Exact-form GELU 0.5 v (1 + erf(v / sqrt 2)).  erf through the rational approximation 7.1.26 of
// Abramowitz & Stegun (|error| <= 1.5e-7, far below the bf16 / fp32 rounding of the result) on the
// native reciprocal and exp2 units instead of the branchy library erff: this runs once per output
// element of the FFN up-projection.
__device__ __forceinline__ float gelu_erf(float v) {
  // GELU(v) = v Phi(v) = max(v, 0) - |v| h,  h = erfc(|v| / sqrt 2) / 2 = (poly(t) / 2) e^(-v^2 / 2),
  // t = 1 / (1 + p |v| / sqrt 2): the 1/2 and the 1/sqrt 2 are folded into the constants
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f * 0.70710678118654752f, fabsf(v), 1.0f));
  float poly = fmaf(0.5f * 1.061405429f, t, 0.5f * -1.453152027f);
  poly = fmaf(poly, t, 0.5f * 1.421413741f);
  poly = fmaf(poly, t, 0.5f * -0.284496736f);
  poly = fmaf(poly, t, 0.5f * 0.254829592f);
  poly *= t;
  const float w = v * 0.84932180028801904f;                 // sqrt(log2(e) / 2): e^(-v^2/2) = 2^(-w^2)
  const float h = poly * __builtin_amdgcn_exp2f(-w * w);
  // |v| h with the legacy multiply's 0 * inf = 0: an overflowed accumulator (v = +-inf, h = 0) saturates to
  // +inf / 0 as the erf form does, instead of turning into NaN; NaN stays NaN
  float tail;
  asm("v_mul_legacy_f32 %0, |%1|, %2" : "=v"(tail) : "v"(v), "v"(h));
  return fmaxf(v, 0.0f) - tail;
}

// tanh-form GELU 0.5 v (1 + tanh(z)), z = sqrt(2/pi) (v + 0.044715 v^3), written as v / (1 + e^(-2z)).
__device__ __forceinline__ float gelu_tanh(float v) {
  const float z = 0.7978845608028654f * fmaf(0.044715f * v * v, v, v);
  const float e = __builtin_amdgcn_exp2f(-2.0f * 1.4426950408889634f * z);   // inf for very negative z: v / inf = -0
  return v * __builtin_amdgcn_rcpf(1.0f + e);
}

// Entropy partials of two disjoint column sets of one row, merged in place into the first:
// against the common maximum M, S = sum f_i S_i and T = sum f_i (T_i + (M - m_i) S_i), f_i = e^(m_i - M).
// An empty set is m = -inf, S = T = 0.
__device__ __forceinline__ void entropy_merge(float& m, float& S, float& T, float m2, float S2, float T2) {
  const float M = fmaxf(m, m2);
  if (M == -INFINITY) return;
  const float kLog2e = 1.4426950408889634f;
  const float f1 = __builtin_amdgcn_exp2f((m - M) * kLog2e), f2 = __builtin_amdgcn_exp2f((m2 - M) * kLog2e);
  const float t1 = (m == -INFINITY) ? 0.0f : f1 * fmaf(M - m, S, T);
  const float t2 = (m2 == -INFINITY) ? 0.0f : f2 * fmaf(M - m2, S2, T2);
  S = f1 * S + f2 * S2;
  T = t1 + t2;
  m = M;
}

template <typename T, int MODE>
__device__ __forceinline__ void epilogue_store(const EpiParams<T>& p, int row, int col, float acc) {
  float v = acc + (p.bias ? (float)p.bias[col] : 0.0f);
  if (MODE == EPI_QKV) {
    const int sel = col / p.C;
    const int c = col - sel * p.C;
    if (sel == 0) {
      p.out[(int64_t)row * p.ldo + c] = (T)v;
    } else {
      const int b = row / p.k, s = row - b * p.k;
      if (s >= image_count(p.k_rows, b, p.k)) return;         // a slot past this image's keep count: nothing to append
      const int Pb = image_prior(p.kv_rows, b, p.P);
      const int head = c / p.dh, d = c - head * p.dh;
      const int64_t bh = (int64_t)b * p.heads + head;
      if (sel == 1) p.kc[(bh * p.cap + Pb + s) * p.dh + d] = (T)v;
      else          p.vc[(bh * p.dh + d) * p.cap + Pb + s] = (T)v;
    }
  } else if (MODE == EPI_ATTN_OUT) {
    const int b = row / p.k;
    const int64_t srow = (int64_t)b * p.Ntok + min(max(p.idx[row], 0), p.Ntok - 1);
    if (p.gate) v *= (float)p.gate[(int64_t)b * p.gate_pitch + col];
    p.out[(int64_t)row * p.ldo + col] = (T)(v + (float)p.res[srow * p.C + col]);
  } else if (MODE == EPI_GELU) {
    p.out[(int64_t)row * p.ldo + col] = (T)gelu_erf(v);
  } else if (MODE == EPI_GELU_TANH) {
    p.out[(int64_t)row * p.ldo + col] = (T)gelu_tanh(v);
  } else if (MODE == EPI_PLAIN) {
    p.out[(int64_t)row * p.ldo + col] = (T)v;
  } else {
    if (p.gate) v *= (float)p.gate[(int64_t)(row / p.k) * p.gate_pitch + col];
    p.out[(int64_t)row * p.ldo + col] = (T)(v + (float)p.res[(int64_t)row * p.ldo + col]);
  }
}
