// Unit-length queries and keys (a block variant of the backbones in Sec. 4: cosine-similarity
// attention with a per-head multiplier).  After the QKV projection has written the queries to the
// workspace and appended the keys to the cache, one wave per (kept row, head) rescales both in place:
//   q <- qk_scale[head] * q / max(|q|, 1e-12),   k <- k / max(|k|, 1e-12)
// so that the attention kernel runs unchanged with a score multiplier of 1.  Norms in fp32.  The bf16 kernel
// (head sizes 64 and 128) moves 16 bytes per lane and packs several (row, head) items into a wave.
#include "common.h"
#include "nova_internal.h"

namespace {

constexpr int kWavesPerBlock = 4;
constexpr float kNormFloor = 1e-12f;

template <typename T>
__global__ __launch_bounds__(kWavesPerBlock* NOVA_WAVE) void qk_norm_kernel(
    T* __restrict__ q, T* __restrict__ kc, const float* __restrict__ qk_scale, float q_mult, int M, int k, int C, int heads,
    int dh, int cap, int P, const int32_t* __restrict__ k_rows, const int32_t* __restrict__ kv_rows) {
  const int lane = threadIdx.x & (NOVA_WAVE - 1);
  const int64_t item = (int64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / NOVA_WAVE;   // (row m, head)
  if (item >= (int64_t)M * heads) return;
  const int m = (int)(item / heads), head = (int)(item - (int64_t)m * heads);
  const int b = m / k, s = m - b * k;
  if (s >= image_count(k_rows, b, k)) return;          // a slot past its image's keep count: no key row was appended
  T* qp = q + (int64_t)m * C + head * dh;
  T* kp = kc + (((int64_t)b * heads + head) * cap + image_prior(kv_rows, b, P) + s) * dh;
  float sq = 0.f, sk = 0.f;
  for (int d = lane; d < dh; d += NOVA_WAVE) {
    const float a = (float)qp[d], c = (float)kp[d];
    sq = fmaf(a, a, sq);
    sk = fmaf(c, c, sk);
  }
  const float fq = q_mult * qk_scale[head] / fmaxf(sqrtf(wave_sum(sq)), kNormFloor);
  const float fk = 1.0f / fmaxf(sqrtf(wave_sum(sk)), kNormFloor);
  for (int d = lane; d < dh; d += NOVA_WAVE) {
    qp[d] = (T)((float)qp[d] * fq);
    kp[d] = (T)((float)kp[d] * fk);
  }
}

// bf16, dh in {64, 128}: 16 bytes per lane, dh / 8 lanes per (row, head), several items per wave
template <int DH>
__global__ __launch_bounds__(kWavesPerBlock* NOVA_WAVE) void qk_norm_bf16_kernel(
    bf16_t* __restrict__ q, bf16_t* __restrict__ kc, const float* __restrict__ qk_scale, float q_mult, int M, int k, int C,
    int heads, int cap, int P, const int32_t* __restrict__ k_rows, const int32_t* __restrict__ kv_rows) {
  constexpr int LPI = DH / 8;                 // lanes per item
  constexpr int IPW = NOVA_WAVE / LPI;        // items per wave
  const int lane = threadIdx.x & (NOVA_WAVE - 1);
  const int sub = lane % LPI;
  const int64_t item = ((int64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / NOVA_WAVE) * IPW + lane / LPI;
  bool live = item < (int64_t)M * heads;         // dead lanes still take part in the shuffles below
  int64_t it = live ? item : 0;
  if (k_rows && (int)(it / heads) % k >= image_count(k_rows, (int)(it / heads) / k, k)) {
    live = false;                                // a slot past its image's keep count: no key row was appended
    it = 0;
  }
  const int m = (int)(it / heads), head = (int)(it - (int64_t)m * heads);
  const int b = m / k, s = m - b * k;
  bf16_t* qp = q + (int64_t)m * C + head * DH + sub * 8;
  // item 0 stands in for dead lanes (loads only); its own key row exists whenever image 0 keeps a token, and
  // otherwise the slot right behind image 0's prior rows is still inside the allocation
  bf16_t* kp = kc + (((int64_t)b * heads + head) * cap + image_prior(kv_rows, b, P) + s) * DH + sub * 8;
  const bf16x8 qv = *reinterpret_cast<const bf16x8*>(qp);
  const bf16x8 kv = *reinterpret_cast<const bf16x8*>(kp);
  float sq = 0.f, sk = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    sq = fmaf((float)qv[e], (float)qv[e], sq);
    sk = fmaf((float)kv[e], (float)kv[e], sk);
  }
#pragma unroll
  for (int o = LPI / 2; o > 0; o >>= 1) {
    sq += __shfl_xor(sq, o, NOVA_WAVE);
    sk += __shfl_xor(sk, o, NOVA_WAVE);
  }
  if (!live) return;
  const float fq = q_mult * qk_scale[head] / fmaxf(sqrtf(sq), kNormFloor);
  const float fk = 1.0f / fmaxf(sqrtf(sk), kNormFloor);
  bf16x8 qo, ko;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    qo[e] = (bf16_t)((float)qv[e] * fq);
    ko[e] = (bf16_t)((float)kv[e] * fk);
  }
  *reinterpret_cast<bf16x8*>(qp) = qo;
  *reinterpret_cast<bf16x8*>(kp) = ko;
}

}  // namespace

hipError_t launch_qk_norm(hipStream_t st, int dtype, void* q, void* kc, const float* qk_scale, float q_mult, int B, int k, int C,
                          int heads, int cap, int P, const int32_t* k_rows, const int32_t* kv_rows) {
  const int M = B * k, dh = C / heads;
  const int64_t items = (int64_t)M * heads;
  const unsigned grid = (unsigned)((items + kWavesPerBlock - 1) / kWavesPerBlock);
  if (dtype == NOVA_BF16 && (dh == 64 || dh == 128)) {
    const int ipb = kWavesPerBlock * (NOVA_WAVE / (dh / 8));            // items per workgroup
    const unsigned gridv = (unsigned)((items + ipb - 1) / ipb);
    if (dh == 64)
      qk_norm_bf16_kernel<64><<<gridv, kWavesPerBlock * NOVA_WAVE, 0, st>>>(
          static_cast<bf16_t*>(q), static_cast<bf16_t*>(kc), qk_scale, q_mult, M, k, C, heads, cap, P, k_rows, kv_rows);
    else
      qk_norm_bf16_kernel<128><<<gridv, kWavesPerBlock * NOVA_WAVE, 0, st>>>(
          static_cast<bf16_t*>(q), static_cast<bf16_t*>(kc), qk_scale, q_mult, M, k, C, heads, cap, P, k_rows, kv_rows);
  } else if (dtype == NOVA_BF16)
    qk_norm_kernel<bf16_t><<<grid, kWavesPerBlock * NOVA_WAVE, 0, st>>>(
        static_cast<bf16_t*>(q), static_cast<bf16_t*>(kc), qk_scale, q_mult, M, k, C, heads, dh, cap, P, k_rows, kv_rows);
  else
    qk_norm_kernel<float><<<grid, kWavesPerBlock * NOVA_WAVE, 0, st>>>(
        static_cast<float*>(q), static_cast<float*>(kc), qk_scale, q_mult, M, k, C, heads, dh, cap, P, k_rows, kv_rows);
  return hipGetLastError();
}
